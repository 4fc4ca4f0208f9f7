// Two-kernel train step for small fp32 networks, where the step is bound by launch latency
// and by dependent phases rather than by arithmetic.
//
// Everything that concerns one sampled experience is independent of the other rows of the
// batch: its slot draw, its gather, the forward pass on s and s', the TD target, and the
// backward pass down to the pre-activation gradients.  Kernel 1 does all of that for two or four
// experiences per workgroup, keeping activations in LDS and streaming the weights through
// 4x4x1 fp32 MFMA (four rows per instruction, so a four-row tile is not padded).  One more
// workgroup of the launch appends the step's new experiences, and a frozen target network gets
// workgroups of its own, which compute max_a Q_target(s', a) a step ahead of the workgroups
// that hold s.  Only the weight gradients reduce over the batch:
// kernel 2 forms them tile by tile and applies the optimizer to each tile as soon as it is
// complete, so gradients never make a round trip through HBM before the update.
//
// Paper: Integration with Reinforcement Learning Algorithm (train step with no host inputs),
// Deep Q-Network Model (update equation), Methods (add, sample).
#include <cstdlib>
#include <cstring>

#include "gather_block.hpp"
#include "mm_f32.hpp"
#include "philox.hpp"
#include "replay_kernels.hpp"
#include "trainer.hpp"

namespace rp {
namespace {

constexpr unsigned int kThreads = kTrainThreads;   // weight kernel
constexpr unsigned int kRowThreads = 1024;         // row kernel: 16 wavefronts
constexpr unsigned int kRows = 4;          // experiences per workgroup of the row kernel ...
constexpr unsigned int kSmallBatch = 512;  // ... and 2 for batches up to this size (no target network):
                                           // measured faster while the workgroups fit the 256 compute units
constexpr unsigned int kSmallBatchSplit = 168;   // the same with a target network (three workgroups per group)
constexpr unsigned int kChunk = 256;       // output columns the workgroup covers per pass
constexpr size_t kRowLdsMax = 160 * 1024;  // dynamic LDS the row kernel may ask for (all of a CU's)
constexpr unsigned int kPadK = 4;          // LDS row padding (floats) against bank conflicts


// Workgroup barrier that orders LDS traffic only.  __syncthreads() also waits for every
// outstanding global load of the wavefront, which would cancel the register prefetch of the
// weights; the row kernel exchanges data between wavefronts through LDS alone.
__device__ __forceinline__ void lds_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}


// A kernel's arguments arrive through the scalar cache, one 64-byte line per miss, and a miss
// costs a few hundred nanoseconds.  Touching every line of the argument block at once, first
// thing, turns a chain of such misses (one per group of fields, as the code reaches them)
// into a single wait.
template <class Args>
__device__ __forceinline__ void touch_kernel_args() {
    const __attribute__((address_space(4))) unsigned int* ka =
        (const __attribute__((address_space(4))) unsigned int*)__builtin_amdgcn_kernarg_segment_ptr();
    unsigned int seen = 0;
#pragma unroll
    for (unsigned int i = 0; i < sizeof(Args) / 4; i += 16) seen |= ka[i];
    asm volatile("" ::"s"(seen));
}

// One 32-bit word of the packed row of experience k of a structure-of-arrays payload.
__device__ __forceinline__ unsigned int payload_word(const Payload& src, unsigned int D,
                                                     unsigned long long k, unsigned int w) {
    if (w < D) return reinterpret_cast<const unsigned int*>(src.s)[k * D + w];
    if (w < 2 * D) return reinterpret_cast<const unsigned int*>(src.s_next)[k * D + w - D];
    if (w == 2 * D) return (unsigned int)src.a[k];
    if (w == 2 * D + 1) return __float_as_uint(src.r[k]);
    if (w == 2 * D + 2) return src.term[k] ? 1u : 0u;
    return 0u;
}
// ... of a new experience of this step
__device__ __forceinline__ unsigned int staged_word(const RowArgs& p, unsigned long long k,
                                                    unsigned int w) {
    return payload_word(p.src, p.D, k, w);
}

// ----------------------------------------------------------------------------------------
// Products of a few activation rows (LDS) with a weight matrix (global, row-major [K x N]).
// On this machine a global load that misses the local L2 takes about 2 us, longer than all
// the arithmetic of a layer, so the row kernel never computes right after loading: a lane
// fetches its whole share of a weight matrix into registers (load_*) one or two phases before
// the matching mma_* consumes it.  A lane owns one output column and the MFMA takes the
// activations of four rows as its broadcast A operand.
//
// "wide" split (N up to 256): a lane owns four adjacent columns, every wavefront covers columns
// 0..255 and K sixteenth w; one load fetches a lane's four columns of one row (16 bytes), the
// widest and, measured, the fastest way to bring a matrix into a compute unit's registers.
// "narrow" split (N up to 64): a lane owns one column, every wavefront covers columns 0..63
// and K sixteenth w.
// ----------------------------------------------------------------------------------------

template <int NR>
__device__ __forceinline__ void load_cols(float (&wr)[NR], const float* __restrict__ W,
                                          unsigned int N, unsigned int col, unsigned int kbeg,
                                          unsigned int kcount) {
    // kbeg and kcount are the same for the whole wavefront: the address of a row is kept in
    // scalar registers (the empty asm pins it there), the lane adds its 32-bit column offset,
    // and the loads of a lane are unconditional.  Rows past kcount re-read the last row: valid
    // memory, finite values, and the products never use them (mma_cols skips k >= kcount).
    // Lanes past the matrix request nothing and hold zeros (their columns are never summed).
    const unsigned int kb = __builtin_amdgcn_readfirstlane(kbeg);
    const unsigned int kc = __builtin_amdgcn_readfirstlane(kcount);
    const unsigned int cb = col * 4u;
    const gbytes base = (gbytes)reinterpret_cast<const char*>(W) + (size_t)kb * N * 4u;
#pragma unroll
    for (int u = 0; u < NR; ++u) wr[u] = 0.f;
    if (col < N) {
#pragma unroll
        for (int u = 0; u < NR; ++u) {
            const unsigned int uu = (unsigned int)u < kc ? (unsigned int)u : kc - 1u;
            gbytes rb = base + (size_t)uu * N * 4u;
            asm volatile("" : "+s"(rb));
            wr[u] = *(const __attribute__((address_space(1))) float*)(rb + cb);
        }
    }
}

// The same for the wide split: wr[u] = W[kbeg + u][col .. col+3], col a multiple of 4.
template <int NR>
__device__ __forceinline__ void load_cols4(f32x4 (&wr)[NR], const float* __restrict__ W,
                                           unsigned int N, unsigned int col, unsigned int kbeg,
                                           unsigned int kcount) {
    const unsigned int kb = __builtin_amdgcn_readfirstlane(kbeg);
    const unsigned int kc = __builtin_amdgcn_readfirstlane(kcount);
    const unsigned int cb = (col + 3u < N ? col : N - 4u) * 4u;
    const gbytes base = (gbytes)reinterpret_cast<const char*>(W) + (size_t)kb * N * 4u;
#pragma unroll
    for (int u = 0; u < NR; ++u) {
        const unsigned int uu = (unsigned int)u < kc ? (unsigned int)u : kc - 1u;
        gbytes rb = base + (size_t)uu * N * 4u;
        asm volatile("" : "+s"(rb));
        wr[u] = *(const __attribute__((address_space(1))) f32x4*)(rb + cb);
    }
}

// acc[mg][v] += sum_{u < kcount} act[mg*4 + v][kbeg + u] * wr[u]   (kcount a multiple of 4)
template <int MG, int NR>
__device__ __forceinline__ void mma_cols(f32x4 (&acc)[MG], const float* act, unsigned int ldk,
                                         unsigned int kbeg, unsigned int kcount,
                                         const float (&wr)[NR]) {
    const float* ap = act + (threadIdx.x & 3u) * ldk + kbeg;
#pragma unroll
    for (int mg = 0; mg < MG; ++mg) acc[mg] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int u4 = 0; u4 < NR; u4 += 4) {
        if ((unsigned int)u4 < kcount) {
#pragma unroll
            for (int mg = 0; mg < MG; ++mg) {
                const f32x4 a = *reinterpret_cast<const f32x4*>(ap + (size_t)mg * 4 * ldk + u4);
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    acc[mg] = __builtin_amdgcn_mfma_f32_4x4x1f32(a[u], wr[u4 + u], acc[mg], 0, 0, 0);
            }
        }
    }
}

template <int VEC> struct ActVec;
template <> struct ActVec<2> { typedef float type __attribute__((ext_vector_type(2))); };
template <> struct ActVec<4> { typedef f32x4 type; };

template <int MG, int NR, int VEC>
__device__ __forceinline__ void mma_cols4(f32x4 (&acc)[MG][4], const float* act, unsigned int ldk,
                                          unsigned int kbeg, unsigned int kcount,
                                          const f32x4 (&wr)[NR]) {
    // MG groups of four activation rows (rows mg*4 .. mg*4+3 of act) share the weights
    typedef typename ActVec<VEC>::type avec;
    const float* ap = act + (threadIdx.x & 3u) * ldk + kbeg;
#pragma unroll
    for (int mg = 0; mg < MG; ++mg)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[mg][j] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int u0 = 0; u0 < NR; u0 += VEC) {
        if ((unsigned int)u0 < kcount) {
#pragma unroll
            for (int mg = 0; mg < MG; ++mg) {
                const avec a = *reinterpret_cast<const avec*>(ap + (size_t)mg * 4 * ldk + u0);
#pragma unroll
                for (int u = 0; u < VEC; ++u)
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        acc[mg][j] = __builtin_amdgcn_mfma_f32_4x4x1f32(a[u], wr[u0 + u][j], acc[mg][j], 0, 0, 0);
            }
        }
    }
}

// part[slice][row0 + v][cc .. cc+3] = acc[.][v] (wide split; `rows` rows per slice, cc a multiple of 4)
__device__ __forceinline__ void store_part4(float* part, unsigned int slice, unsigned int rows,
                                            unsigned int row0, unsigned int pitch, unsigned int cc,
                                            const f32x4 (&acc)[4]) {
#pragma unroll
    for (int v = 0; v < 4; ++v)
        *reinterpret_cast<f32x4*>(part + ((size_t)(slice * rows + row0 + v)) * pitch + cc) =
            f32x4{acc[0][v], acc[1][v], acc[2][v], acc[3][v]};
}

// part[slice][row][cc] = acc; the lane holds rows v = 0..3 of its column cc
template <int MG>
__device__ __forceinline__ void store_part(float* part, unsigned int slice, unsigned int pitch,
                                           unsigned int cc, const f32x4 (&acc)[MG]) {
#pragma unroll
    for (int mg = 0; mg < MG; ++mg)
#pragma unroll
        for (int v = 0; v < 4; ++v)
            part[((size_t)(slice * (MG * 4) + mg * 4 + v)) * pitch + cc] = acc[mg][v];
}

__device__ __forceinline__ float sum_part(const float* part, unsigned int slices,
                                          unsigned int rows, unsigned int pitch, unsigned int row,
                                          unsigned int c) {
    float v = 0.f;
    for (unsigned int s = 0; s < slices; ++s) v += part[((size_t)(s * rows + row)) * pitch + c];
    return v;
}

// NR1: rows of W1 a lane holds (Dp / 4, 8 or 16).
// R: experiences per workgroup, 4 or 2.  A workgroup's 2 R rows (R states s, then R states s')
// form R / 2 groups of four MFMA rows.  Every workgroup fetches all the weights whatever R is,
// so R = 2 halves a workgroup's products at twice the workgroups: the choice for batches that
// leave most compute units idle anyway.
//
// SPLIT: the frozen target network in workgroups of its own.  Workgroups come in threes for R
// experiences (numbers 3 j, 3 j + 1, 3 j + 2; lower numbers are dispatched first):
//   3 j      ends at once when a table that the previous launch filled holds this step's
//            max_a Q_target(s', a) for all of its experiences; otherwise it sends their states s'
//            through the target network now and hands the maxima over;
//   3 j + 1  does everything for the states s of THIS step, and takes the maxima from the table
//            or, for entries that are not valid for this step, from workgroup 3 j, for which it
//            waits (a bounded time);
//   3 j + 2  sends the states s' of the NEXT step's sample (a function of seed, step and ring
//            size alone) through the target network and fills the table for the next launch,
//            when the host says the target network stays as it is until then.
// Each workgroup then fetches one network's weights and multiplies one group of four rows, like
// a workgroup of the step without a target network, and they run side by side on different
// compute units.  A table entry carries what it was computed for (sampling step, experiences ever
// added, Adam steps, a count of calls that changed weights from outside): it is valid when those
// are this step's.  Its row was read from the ring as it will be at that step: rows this step
// appends come from the payload, rows the next step will overwrite make the entry invalid.
constexpr unsigned int kNowSide = 0, kMainSide = 1, kAheadSide = 2;
constexpr unsigned int kAheadWords = 8;   // step, total, Adam steps (two words each), outside changes, maximum
template <bool SPLIT, int NR1, int R>
__global__ __launch_bounds__(kRowThreads) void fused_rows_kernel(RowArgs p) {
    static_assert(R == 4 || R == 2, "experiences per workgroup (split: per three workgroups)");
    constexpr unsigned int NRW = SPLIT ? 4 : 2 * R;  // rows of a workgroup
    constexpr int MG = NRW / 4;                      // groups of four rows
    constexpr unsigned int PR = NRW;                 // rows of its MFMA groups
    extern __shared__ float lds[];
    touch_kernel_args<RowArgs>();
    const unsigned int wg = SPLIT ? blockIdx.x / 3u : blockIdx.x;
    const unsigned int side = SPLIT ? blockIdx.x - 3u * wg : kMainSide;   // (uniform over the workgroup)
    const bool target_side = side != kMainSide;
    const bool ahead_side = SPLIT && side == kAheadSide;
    if (wg * R >= p.B) {
        // Extra workgroups, after those of the batch.  First (when the trainer appends at all): the
        // one that writes the step's new experiences into the ring.  No workgroup reads those
        // slots from the ring in this launch (they take such rows from the payload), so nothing
        // waits for it; it has compute units to itself, and a payload in host memory, which takes
        // microseconds to arrive, holds up none of the batch's workgroups.
        const unsigned int extra = blockIdx.x - (SPLIT ? 3u : 1u) * ((p.B + R - 1u) / R);
        if (p.append_group && extra == 0) {
            const unsigned long long cap = p.g.capacity, n = p.n_append;
            const unsigned int rw = p.g.row_bytes >> 2;
            for (unsigned long long e = threadIdx.x; e < n * rw; e += kRowThreads) {
                const unsigned long long k = e / rw;
                const unsigned int w = (unsigned int)(e - k * rw);
                unsigned long long slot = p.head + k;
                if (slot >= cap) slot -= cap;
                reinterpret_cast<unsigned int*>(p.g.rows + slot * p.g.row_bytes)[w] = staged_word(p, k, w);
            }
            return;
        }
        // then that of a replay that samples without duplicates: the next step's slots
        const unsigned long long ns = p.step + 1;
        unsigned int* dst = p.pre + ((ns & 1u) ? p.pre_stride : 0u);
        for (unsigned int i = threadIdx.x; i < p.B; i += kRowThreads)
            dst[4 + i] = distinct_draw(p.seed, ns, i, p.next_size);
        if (threadIdx.x == 0) {
            dst[0] = (unsigned int)ns;
            dst[1] = (unsigned int)(ns >> 32);
            dst[2] = p.next_size;
        }
        return;
    }
    const unsigned int tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const unsigned int D = p.D, Dp = p.Dp, H = p.H, A = p.A, Ap = p.Ap;
    const unsigned int ldx = Dp + kPadK, ldh = H + kPadK, ldq = Ap + kPadK;
    float* Xs = lds;                      // [8][ldx]  rows 0..R-1 = s, R..2R-1 = s' (laid out for R = 4)
    float* H1s = Xs + 8 * ldx;            // [8][ldh]
    float* H2s = H1s + 8 * ldh;           // [8][ldh]
    float* Qs = H2s + 8 * ldh;            // [8][ldq]
    float* dZs = Qs + 8 * ldq;            // [4][ldh]
    float* part = dZs + 4 * ldh;          // [16][8][256] or [16][8][64]
    float* b1s = part + 16 * 8 * kChunk;  // [H]   (layer 1's biases stay in registers: unused)
    float* b2s = b1s + H;                 // [H]
    float* b3s = b2s + H;                 // [Ap]
    unsigned int* meta = reinterpret_cast<unsigned int*>(b3s + Ap);   // [4][4]
    float* gs = reinterpret_cast<float*>(meta + 16);                 // [4]
    unsigned int* ahead_s = reinterpret_cast<unsigned int*>(gs + 4); // [4][8]  split: this step's table entries
    float* qn_s = reinterpret_cast<float*>(ahead_s + 4 * kAheadWords);   // [4][64] and their rows Q_target(s', .)
    unsigned int* idle_s = reinterpret_cast<unsigned int*>(qn_s + 4 * 64);   // [1]  split: nothing to do for this workgroup

    const float* wsrc = target_side ? p.wt : p.w;
    const float* W1 = wsrc + p.oW1;
    const float* W2 = wsrc + p.oW2;
    const float* W3 = wsrc + p.oW3;
    // wide split (layer 2 and backward): K sixteenths
    const unsigned int cc = 4u * lane, ks = wave;
    const unsigned int q2 = H >> 4;
    // narrow split
    const unsigned int s3 = H >> 4;                 // K sixteenth of layer 3

    // ---- phase 0.  Fetching the weights is what the kernel waits for longest (the rate at which
    // a compute unit takes in data bounds it), so the request stream never pauses: most
    // wavefronts queue their share of W2 (and W3) from the first instruction on, while a few
    // draw and gather the sample and run layer 1 (the ring and trainer state before this step
    // come as arguments, the host mirrors them exactly, so the draw needs no memory access).
    f32x4 w2r[16];
    float w3r[16];
    f32x4 acc2[MG];
    // layer 3's weights can be requested with W2 by the wavefronts that have no part in
    // layer 1 (two experiences per workgroup: the registers hold them next to layer 2's sums)
    constexpr bool W3_EARLY = MG == 1;          // (two groups of rows: no room)
    constexpr unsigned int NL1 = 4u;            // wavefronts in layer 1
    const unsigned long long cap = p.g.capacity;
    const unsigned long long head = p.head;
    const unsigned long long step = p.step + (ahead_side ? 1u : 0u);   // the step whose sample this workgroup takes
    const unsigned long long n = p.n_append;
    const unsigned int size = ahead_side ? p.next_size : p.size_after;
    const unsigned int i0 = wg * R;
    const unsigned int nrows = min((unsigned int)R, p.B - i0);
    // word j of the table entry that is valid for this step (next: for the step after it)
    auto key_word = [&](unsigned int j, bool next) {
        const unsigned long long st = p.step + (next ? 1u : 0u), tot = next ? p.next_total_after : p.total_after,
                                 ad = p.adam_t_after + (next ? 1u : 0u);
        return j == 0 ? (unsigned int)st : j == 1 ? (unsigned int)(st >> 32) : j == 2 ? (unsigned int)tot
             : j == 3 ? (unsigned int)(tot >> 32) : j == 4 ? (unsigned int)ad : j == 5 ? (unsigned int)(ad >> 32)
             : p.epoch;
    };
    if constexpr (SPLIT) {
        if (ahead_side && !p.ahead_on) return;
        if (side == kNowSide) {
            // nothing to do when the table holds this step's values for all of this workgroup's rows
            // (the first wavefront holds all 8 x 4 words)
            if (wave == 0) {
                bool ok = !p.from_batch;
                if (ok && lane < kAheadWords * nrows) {
                    const unsigned int j = lane & (kAheadWords - 1u);
                    const unsigned int word =
                        p.ahead[((size_t)(p.step & 1u) * p.B + i0 + lane / kAheadWords) * kAheadWords + j];
                    ok = j == kAheadWords - 1u || word == key_word(j, false);
                }
                const bool all = __ballot(ok) == ~0ull;
                if (lane == 0) *idle_s = all ? 1u : 0u;
            }
            __syncthreads();
            if (*idle_s) return;
        }
    }
    // words of a sampled row this workgroup needs: all 2 D + 3, or s and (a, r, terminal), or s'
    const unsigned int words = SPLIT ? (target_side ? D : D + 3u) : 2 * D + 3;

    // The state that follows this step is known up front (the host mirrors it exactly): one
    // thread stores it for the kernels and calls that read it later, off everyone's critical path.
    if (wg == 0 && side == kMainSide && tid == kRowThreads - 1) {
        unsigned long long h = head + n;
        if (h >= cap) h -= cap;
        p.g.state->head = h;
        p.g.state->size = p.size_after;
        p.g.state->total = p.total_after;
        p.ctr->adam_t = p.adam_t_after;
        p.ctr->c1 = p.c1_after;
        p.ctr->c2 = p.c2_after;
    }

    {
        // ---- layer 1: wavefronts 0..3 take it on their own, each for
        // 64 output columns over the whole K, from a private copy of the sample: no partial sums
        // and no barrier before layer 2's, so nothing here waits for the wavefronts that are still
        // queueing their requests for W2.  Each of the four draws and gathers the (few) sampled
        // words itself, and they share publishing them: wavefront 1 the action / reward / terminal
        // words, the others the states, a pass each.
        constexpr int MGF = MG;                         // groups of four rows each of them takes
        const unsigned int wq = wave & 3u;
        if (wave < NL1) {
            // one draw per row, in the lane of that row: first of all, the sampled words take
            // longest to arrive
            unsigned int myslot = 0;
            if (lane < nrows) {
                if (p.from_batch) {
                    myslot = i0 + lane;
                } else {
                    // (slots drawn a step ahead: only for replays that sample without duplicates,
                    // which have no table of target values a step ahead)
                    const unsigned int* ahead = p.pre ? p.pre + ((step & 1u) ? p.pre_stride : 0u) : nullptr;
                    if (ahead && ahead[0] == (unsigned int)step && ahead[1] == (unsigned int)(step >> 32) &&
                        ahead[2] == size)
                        myslot = ahead[4 + i0 + lane];   // drawn during the previous step
                    else
                        myslot = batch_draw(p.g.sampling, p.seed, step, i0 + lane, size);
                }
            }
            // D <= 4 NR1: at most 8 NR1 + 3 words per row (split: 4 NR1 + 3)
            constexpr int NPASS = (R * ((SPLIT ? 4 : 8) * NR1 + 3) + 63) / 64;
            unsigned int gv[NPASS], gsl[NPASS];
            // word `wl` of this workgroup's share of a row -> word of the row [s | s' | a r terminal]
            auto row_word = [&](unsigned int wl) {
                return !SPLIT ? wl : target_side ? wl + D : wl < D ? wl : wl + D;
            };
#pragma unroll
            for (int pass = 0; pass < NPASS; ++pass) {
                const unsigned int e = lane + 64u * pass;
                const unsigned int r = min(e / words, (unsigned int)R - 1u), w = row_word(e - r * words);
                const unsigned int slot = __shfl(myslot, (int)r, 64);
                gv[pass] = 0u;
                gsl[pass] = slot;
                if (e < nrows * words) {
                    if (p.from_batch) {
                        gv[pass] = payload_word(p.batch, D, i0 + r, w);
                    } else {
                        unsigned long long off = (unsigned long long)slot + cap - head;
                        if (off >= cap) off -= cap;
                        gv[pass] = off < n ? staged_word(p, off, w)
                                           : reinterpret_cast<const unsigned int*>(
                                                 p.g.rows + (unsigned long long)slot * p.g.row_bytes)[w];
                    }
                }
            }
            // W1: the wavefront covers columns 64 w .. 64 w + 63 as 16 groups of four adjacent
            // columns times 4 quarters of K (NR1 rows each).  Lane l = 16 q + 4 kq + i: column
            // group 4 q + i, K quarter kq -- the four lanes of an MFMA block share their kq (they
            // exchange operands), the four quarters of a column sit in one DPP row.
            const unsigned int kq = (lane >> 2) & 3u;
            const unsigned int ccf = 64u * wq + 4u * (4u * (lane >> 4) + (lane & 3u));
            const bool colf = ccf < H;   // (H is a multiple of 64: all four columns or none)
            f32x4 w1x[NR1];
            {
                const unsigned int loff = (((unsigned int)NR1 * kq) * H + (colf ? ccf : H - 4u)) * 4u;
                const gbytes base = (gbytes)reinterpret_cast<const char*>(W1);
#pragma unroll
                for (int u = 0; u < NR1; ++u) {
                    gbytes rb = base + (size_t)u * H * 4u;
                    asm volatile("" : "+s"(rb));
                    w1x[u] = *(const __attribute__((address_space(1))) f32x4*)(rb + loff);
                }
            }
            const f32x4 b1f = *reinterpret_cast<const f32x4*>(wsrc + p.ob1 + (colf ? ccf : H - 4u));
            // the private copy (in the partial-sum buffer, which nothing uses before layer 2)
            float* Xp = part + wave * (PR * ldx);
            for (unsigned int e = lane; e < PR * ldx; e += 64u) Xp[e] = 0.f;
            // (word 3 of a row's four: for the step after this one, whether the next step's
            // append overwrites the row, so that its content is not known yet)
            unsigned int unknown = 0;
            if constexpr (SPLIT) {
                unsigned long long off = (unsigned long long)__shfl(myslot, (int)((lane >> 2) & 3u), 64) + cap - head;
                if (off >= cap) off -= cap;
                // (position counted from where the next append starts; on a ring shorter than two
                // appends that range laps into this step's own)
                const unsigned long long off2 = off >= n ? off - n : off + cap - n;
                unknown = ahead_side && (lane >> 2) < nrows && off2 < n;
            }
            if (wave == 1 && lane < 16 && ((lane >> 2) >= nrows || (lane & 3u) == 3u)) meta[lane] = unknown;
#pragma unroll
            for (int pass = 0; pass < NPASS; ++pass) {
                const unsigned int e = lane + 64u * pass;
                if (e < nrows * words) {
                    const unsigned int r = e / words, w = row_word(e - r * words);
                    const unsigned int i = i0 + r;
                    const unsigned int val = gv[pass];
                    if (w < D) {
                        Xp[r * ldx + w] = __uint_as_float(val);
                        if (wave == (pass % 3 == 0 ? 0u : pass % 3 == 1 ? 2u : 3u))
                            p.X[(size_t)i * Dp + w] = __uint_as_float(val);
                    } else if (w < 2 * D) {
                        Xp[((SPLIT ? 0u : (unsigned int)R) + r) * ldx + w - D] = __uint_as_float(val);
                    } else if (wave == 1) {
                        meta[r * 4 + (w - 2 * D)] = val;
                        if (w == 2 * D) {
                            p.act[i] = (int)val;
                            p.idx[i] = gsl[pass];
                        } else if (w == 2 * D + 1) {
                            p.rew[i] = __uint_as_float(val);
                        } else {
                            p.term[i] = (unsigned char)val;
                        }
                    }
                }
            }
            // (a wavefront's LDS operations complete in order: its copy is there)
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            f32x4 accf[MGF][4];
            {
                const float* ap = Xp + (lane & 3u) * ldx + (unsigned int)NR1 * kq;
#pragma unroll
                for (int mg = 0; mg < MGF; ++mg)
#pragma unroll
                    for (int j = 0; j < 4; ++j) accf[mg][j] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int u0 = 0; u0 < NR1; u0 += 4)
#pragma unroll
                    for (int mg = 0; mg < MGF; ++mg) {
                        const f32x4 av = *reinterpret_cast<const f32x4*>(ap + (size_t)mg * 4 * ldx + u0);
#pragma unroll
                        for (int u = 0; u < 4; ++u)
#pragma unroll
                            for (int j = 0; j < 4; ++j)
                                accf[mg][j] = __builtin_amdgcn_mfma_f32_4x4x1f32(av[u], w1x[u0 + u][j],
                                                                                 accf[mg][j], 0, 0, 0);
                    }
            }
            // sum the four K quarters (lanes 4 apart within a DPP row), then lane kq takes row kq
#pragma unroll
            for (int mg = 0; mg < MGF; ++mg) {
                f32x4 hv = b1f;
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        float x = accf[mg][j][v];
                        x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x128, 0xf, 0xf, false));
                        x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x124, 0xf, 0xf, false));
                        if ((unsigned int)v == kq) hv[j] += x;
                    }
#pragma unroll
                for (int j = 0; j < 4; ++j) hv[j] = hv[j] > 0.f ? hv[j] : 0.f;
                const unsigned int row = mg * 4 + kq;
                if (colf) {
                    *reinterpret_cast<f32x4*>(H1s + row * ldh + ccf) = hv;
                    if (row < nrows && !target_side)
                        *reinterpret_cast<f32x4*>(p.H1 + (size_t)(i0 + row) * H + ccf) = hv;
                }
            }
            load_cols4<16>(w2r, W2, H, cc, ks * q2, q2);
        } else {
            // (main side, the four wavefronts of the TD phase: this step's table entries and rows,
            // requested ahead of everything else and parked in LDS once they are there)
            unsigned int aw = 0;
            float aq = 0.f;
            const bool looks_up = SPLIT && !target_side && wave >= 12 && wave - 12u < nrows && !p.from_batch;
            if (looks_up) {
                const size_t e = (size_t)(p.step & 1u) * p.B + i0 + (wave - 12u);
                aw = p.ahead[e * kAheadWords + (lane & (kAheadWords - 1u))];
                if (lane < Ap) aq = p.qn_ahead[e * Ap + lane];
            }
            load_cols4<16>(w2r, W2, H, cc, ks * q2, q2);
            if constexpr (W3_EARLY) load_cols<16>(w3r, W3, Ap, lane, wave * s3, s3);
            if (SPLIT && wave >= 12) {
                if (lane < kAheadWords) ahead_s[(wave - 12u) * kAheadWords + lane] = looks_up ? aw : ~0u;
                qn_s[(wave - 12u) * 64u + lane] = aq;
            }
            // the other biases: the four wavefronts after layer 1's
            const unsigned int t4 = tid - 64u * NL1;
            if (t4 < H) b2s[t4] = wsrc[p.ob2 + t4];
            if (t4 < Ap) b3s[t4] = wsrc[p.ob3 + t4];
        }
        lds_barrier();
    }

    // ---- layer 2.  From here on the fetch of W2^T (for the backward pass, into the registers
    // that layer 2 frees) is the long pole: a wavefront that requests its share stalls for about
    // half a microsecond while its SIMD's load path is busy, so each wavefront does it in a
    // phase in which the others have all the work: wavefronts 8..15 during layer 2's sums
    // (wavefronts 0..7), wavefronts 0..7 during layer 3's sums and the TD phase (12..15).
    {
        f32x4 acc8[MG][4];
        mma_cols4<MG, 16, 4>(acc8, H1s, ldh, ks * q2, q2, w2r);
#pragma unroll
        for (int mg = 0; mg < MG; ++mg) store_part4(part, ks, NRW, 4 * mg, kChunk, cc, acc8[mg]);
    }
    // The accumulators are free: layer 3's weights are requested, and ...
    if (!W3_EARLY || wave < NL1) load_cols<16>(w3r, W3, Ap, lane, wave * s3, s3);
    // ... the column of W3 that the backward pass of each row needs: W3[k][a_r], one per thread
    float w3sel = 0.f;
    {
        const unsigned int r = tid / H, k = tid - r * H;
        if (r < nrows && !target_side) {
            unsigned int ai = meta[r * 4 + 0];
            if (ai >= A) ai = A - 1;  // an out-of-range action must not turn into a wild address
            w3sel = W3[(size_t)k * Ap + ai];
        }
    }
    lds_barrier();
    if (wave < 8) {
        // four adjacent columns of one row per thread, 16-byte LDS accesses
        for (unsigned int e = tid; e < NRW * (H >> 2); e += 512u) {
            const unsigned int row = e / (H >> 2), c = (e - row * (H >> 2)) * 4u;
            f32x4 v = *reinterpret_cast<const f32x4*>(b2s + c);
            for (unsigned int sl = 0; sl < 16; ++sl)
                v += *reinterpret_cast<const f32x4*>(part + ((size_t)(sl * NRW + row)) * kChunk + c);
#pragma unroll
            for (int j = 0; j < 4; ++j) v[j] = v[j] > 0.f ? v[j] : 0.f;
            *reinterpret_cast<f32x4*>(H2s + row * ldh + c) = v;
            if (row < nrows && !target_side) *reinterpret_cast<f32x4*>(p.H2 + (size_t)(i0 + row) * H + c) = v;
        }
    } else if (!target_side) {
        load_cols4<16>(w2r, p.w2t, H, cc, ks * q2, q2);
    }
    lds_barrier();

    // ---- layer 3 (narrow split: 16 K slices, columns 0..63)
    mma_cols<MG, 16>(acc2, H2s, ldh, wave * s3, s3, w3r);
    store_part<MG>(part, wave, 64, lane, acc2);
    lds_barrier();

    // ---- Q values (sums of the partial products), TD target, loss term, dL/dQ: wavefront
    // 12 + r takes rows r (s) and R + r (s'), one action per lane (A <= 64).  What it has to
    // store to global memory waits until the next phase: right now the load path is busy with
    // the other wavefronts' requests and a store would queue up behind them.
    float td_qs = 0.f, td_qn = 0.f, td_y = 0.f, td_d = 0.f, td_li = 0.f, td_gr = 0.f;
    unsigned int td_ai = 0;
    bool td_hit = false;   // split: the table held this step's value for the row
    if (wave >= 12) {
        const unsigned int r = wave - 12u;
        if (r < (unsigned int)R && lane < Ap) {
            td_qs = sum_part(part, 16, NRW, 64, r, lane) + b3s[lane];
            if constexpr (!SPLIT) td_qn = sum_part(part, 16, NRW, 64, R + r, lane) + b3s[lane];
        }
        if (SPLIT && target_side) {
            if (r < nrows) {
                const unsigned int i = i0 + r;
                const float best = wave_max(lane < A ? td_qs : -INFINITY);
                if (ahead_side) {
                    // Q_target(s', .) of this row and its maximum for the next step, with what they hold for
                    const size_t e = (size_t)(step & 1u) * p.B + i;
                    const bool known = meta[r * 4 + 3] == 0u;
                    if (lane < Ap) p.qn_ahead[e * Ap + lane] = td_qs;
                    if (lane < kAheadWords)
                        p.ahead[e * kAheadWords + lane] = lane == kAheadWords - 1u ? __float_as_uint(best)
                                                          : known ? key_word(lane, true) : ~0u;
                } else {
                    // ... for this step, handed over in one 8-byte word that carries this launch's
                    // number (value and tag arrive together or not at all)
                    if (lane < Ap) p.Q[((size_t)p.B + i) * Ap + lane] = td_qs;
                    if (lane == 0)
                        __hip_atomic_store(p.handoff + i, ((unsigned long long)p.seq << 32) | __float_as_uint(best),
                                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            }
        } else if (r < nrows) {
            float best;
            if constexpr (SPLIT) {
                const unsigned int j = lane & (kAheadWords - 1u);
                td_hit = __ballot(j == kAheadWords - 1u || ahead_s[r * kAheadWords + j] == key_word(j, false)) == ~0ull;
            }
            if (SPLIT && td_hit) {
                best = __uint_as_float(ahead_s[r * kAheadWords + kAheadWords - 1u]);
                td_qn = qn_s[r * 64u + lane];
            } else if constexpr (SPLIT) {
                // wait for the other workgroup of the pair: it was dispatched before this one and
                // waits for nothing, so the word arrives; the time limit only guards against a
                // launch that breaks that order (then the step is marked as failed)
                unsigned long long word = 0;
                if (lane == 0) {
                    const long long t0 = wall_clock64();
                    bool there;
                    do {
                        word = __hip_atomic_load(p.handoff + i0 + r, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        there = (unsigned int)(word >> 32) == p.seq_wait;
                    } while (!there && wall_clock64() - t0 < p.handoff_ticks);
                    if (!there) {
                        p.ctr->handoff_missed = 1u;
                        word = 0;
                    }
                }
                best = __uint_as_float((unsigned int)__shfl(word, 0, 64));
            } else {
                best = wave_max(lane < A ? td_qn : -INFINITY);
            }
            td_ai = meta[r * 4 + 0];
            if (td_ai >= A) td_ai = A - 1;
            const float q = __shfl(td_qs, (int)td_ai, 64);
            td_y = __uint_as_float(meta[r * 4 + 1]) + (meta[r * 4 + 2] ? 0.f : p.gamma * best);
            td_d = td_y - q;
            float slope;
            if (p.loss_kind == RP_MSE || fabsf(td_d) <= 1.f) {
                td_li = 0.5f * td_d * td_d;
                slope = td_d;
            } else {
                td_li = fabsf(td_d) - 0.5f;
                slope = td_d > 0.f ? 1.f : -1.f;
            }
            td_gr = -slope / (float)p.B;
            if (lane == 0) gs[r] = td_gr;
        }
    } else if (wave < 8 && !target_side) {
        load_cols4<16>(w2r, p.w2t, H, cc, ks * q2, q2);
    }
    if (target_side) return;   // (the whole workgroup: nothing after this concerns s')
    lds_barrier();
    if (wave >= 12 && wave - 12u < nrows) {
        const unsigned int i = i0 + wave - 12u;
        if (lane < Ap) {
            p.Q[(size_t)i * Ap + lane] = td_qs;
            if (!SPLIT || td_hit) p.Q[((size_t)p.B + i) * Ap + lane] = td_qn;
            p.dQ[(size_t)i * Ap + lane] = lane == td_ai ? td_gr : 0.f;
        }
        if (lane == 0) {
            if (SPLIT && i == 0) p.ctr->from_table = td_hit ? 1u : 0u;
            p.y[i] = td_y;
            p.delta[i] = td_d;
            p.lossi[i] = td_li;
        }
    }
    // dZ2[r][k] = dQ[r][a_r] * W3[k][a_r] * 1[H2[r][k] > 0]
    {
        const unsigned int r = tid / H, k = tid - r * H;
        if (r < 4) {
            float v = 0.f;
            if (r < nrows && H2s[r * ldh + k] > 0.f) v = gs[r] * w3sel;
            dZs[r * ldh + k] = v;
            if (r < nrows) p.dZ2[(size_t)(i0 + r) * H + k] = v;
        }
    }
    lds_barrier();

    // ---- dZ1 = (dZ2 W2^T) masked by the first ReLU
    f32x4 accw[1][4];
    mma_cols4<1, 16, 4>(accw, dZs, ldh, ks * q2, q2, w2r);
    store_part4(part, ks, 4, 0, kChunk, cc, accw[0]);
    lds_barrier();
    for (unsigned int e = tid; e < nrows * H; e += kRowThreads) {
        const unsigned int r = e / H, c = e - r * H;
        float v = sum_part(part, 16, 4, kChunk, r, c);
        if (!(H1s[r * ldh + c] > 0.f)) v = 0.f;
        p.dZ1[(size_t)(i0 + r) * H + c] = v;
    }

}

// ----------------------------------------------------------------------------------------
// Kernel 2: weight gradients and optimizer.  A job is one layer: G[M x N] = Act^T Err with
// Act [B x M] and Err [B x N]; the bias gradient is the column sum of Err.
// ----------------------------------------------------------------------------------------
struct WJob {
    const float* act;   // [B x M]
    unsigned int lda;
    const float* err;   // [B x N]
    unsigned int ldb;
    unsigned int M, N;
    unsigned int w_off, ldw, b_off;
    float* wT;          // transposed copy of the weight matrix to maintain ([N x M]) or null
    unsigned int tiles_n, tile_begin;
};

struct WArgs {
    WJob job[3];
    unsigned int B, n_tiles;
    float *w, *g, *m, *v;
    unsigned int opt;
    float lr, beta1, beta2, eps;
    TrainCounters* ctr;
    const float* lossi;
    unsigned int grad_only_job;   // a job whose update another kernel makes (dueling head), or ~0
    // A dueling head of up to 32 actions is updated here: the tiles of job fold_job (else ~0)
    // hold the gradient of the plain output layer the head amounts to, one whole row of it per
    // 32 lanes, which is all the head's own update needs.  The head's parameters are rows of
    // 1 + head_A entries (state value first) starting at entry head_off of w, g, m, v, wt.
    unsigned int fold_job, head_A, head_off;
    float* wt;                    // frozen target network, synced when Adam's t is a multiple of
    unsigned int sync_every;      // sync_every (0: never)
    // 1: the launch whose last tile writes the step's loss and advances the step count (one
    // launch per train step; a step's other launch of tiles leaves both alone)
    unsigned int closes_step;
};

constexpr unsigned int kTM = 32, kTN = 32, kTK = 128;

// Sum over the 16 lanes of a DPP row (lanes 16 q .. 16 q + 15), returned in each of them.
__device__ __forceinline__ float row16_sum(float v) {
    // row_ror:8, 4, 2, 1 -- rotations within a row of 16 lanes
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x128, 0xf, 0xf, false));
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x124, 0xf, 0xf, false));
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x122, 0xf, 0xf, false));
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x121, 0xf, 0xf, false));
    return v;
}

// Element k of a parameter array, addressed as the array's (uniform) base plus a 32-bit byte
// offset: one address register per access instead of 64-bit arithmetic per lane.  (The arrays
// are far smaller than 4 GiB.)
__device__ __forceinline__ float ldw(const float* base, unsigned int k) {
    return *(const __attribute__((address_space(1))) float*)((gbytes)reinterpret_cast<const char*>(base) + k * 4u);
}
__device__ __forceinline__ void stw(float* base, unsigned int k, float v) {
    typedef __attribute__((address_space(1))) char* gwbytes;
    *(__attribute__((address_space(1))) float*)((gwbytes)reinterpret_cast<char*>(base) + k * 4u) = v;
}

// One optimizer update of parameter k with gradient gk, from values loaded earlier.
// r1 = 1 / (1 - beta1^t), r2 = 1 / (1 - beta2^t); sync: this step also refreshes the target network.
__device__ __forceinline__ float opt_apply(const WArgs& p, unsigned int k, float gk, float wk,
                                           float mk, float vk, float r1, float r2, bool grad_only,
                                           bool sync) {
    stw(p.g, k, gk);
    if (grad_only) return wk;
    if (p.opt == RP_SGD) {
        wk -= p.lr * gk;
    } else {
        mk = p.beta1 * mk + (1.f - p.beta1) * gk;
        vk = p.beta2 * vk + (1.f - p.beta2) * gk * gk;
        stw(p.m, k, mk);
        stw(p.v, k, vk);
        // hardware square root and reciprocal (1 ulp each): the quotient is good to a few parts
        // in 1e7, far inside what the update's own rounding leaves
        wk -= p.lr * (mk * r1) * __builtin_amdgcn_rcpf(__builtin_amdgcn_sqrtf(vk * r2) + p.eps);
    }
    stw(p.w, k, wk);
    if (sync) stw(p.wt, k, wk);
    return wk;
}

// A workgroup owns a 32 x 32 tile of one layer's weight matrix (every matrix here is a whole
// number of tiles) and wavefront w its 16 x 16 quarter (w >> 1, w & 1): it reduces the outer
// products over the batch with 16x16x4 fp32 MFMA, 128 batch rows per pass, adds the bias
// gradient when it sits on tile row 0 (the column sums of its error operands), and applies
// the optimizer to what it holds.  The MFMA operands go from global
// memory straight into the registers the instruction reads them from (lane l: batch row
// 4t + l/16 of step t, column l%16 of the quarter -- 64-byte runs), all 64 loads of a pass
// requested before the first use; nothing passes through LDS and no wavefront waits for another.
// FOLD: the variant that also updates a dueling head (the tiles of job fold_job).
// block: the workgroup's number among the launch's tiles.
template <bool FOLD>
__device__ __forceinline__ void weights_tile(const WArgs& p, unsigned int block) {
    const unsigned int tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const unsigned int l16 = lane & 15u, lq = lane >> 4;
    const unsigned int wr = wave >> 1, wc = wave & 1u;
    unsigned int j = 0;
    if (block >= p.job[1].tile_begin) j = 1;
    if (block >= p.job[2].tile_begin) j = 2;
    const WJob jb = j == 0 ? p.job[0] : j == 1 ? p.job[1] : p.job[2];
    const unsigned int tile = block - jb.tile_begin;
    const unsigned int m0 = (tile / jb.tiles_n) * kTM, n0 = (tile % jb.tiles_n) * kTN;
    // this lane's outputs: rows mm .. mm+3 of column nn
    const unsigned int nn = n0 + 16u * wc + l16;
    const unsigned int mm = m0 + 16u * wr + 4u * lq;
    const bool bias_wave = m0 == 0 && wr == 0;
    const bool do_bias = bias_wave && lq == 0;

    // operands of one pass: a[t] = Act[b0 + 4t + lq][m0 + 16 wr + l16], b[t] = Err[same row][nn].
    // The address of a step's four rows is a scalar and the lane adds its byte offset within
    // them.  A step past the batch contributes zeros without touching memory; the one step
    // that straddles its end (batch not a multiple of 4) reads the last row in the lanes past
    // it and zeroes them.
    constexpr int kSteps = kTK / 4;
    float a[kSteps], b[kSteps];
    const unsigned int ca = (m0 + 16u * wr + l16) * 4u, cb = nn * 4u;
    const unsigned int la = lq * jb.lda * 4u + ca, lb = lq * jb.ldb * 4u + cb;
    const unsigned int lqc = min(lq, (p.B - 1u) & 3u);
    const unsigned int la_c = lqc * jb.lda * 4u + ca, lb_c = lqc * jb.ldb * 4u + cb;
    auto load_pass = [&](unsigned int b0) {
        const gbytes abase = (gbytes)reinterpret_cast<const char*>(jb.act) + (size_t)b0 * jb.lda * 4u;
        const gbytes bbase = (gbytes)reinterpret_cast<const char*>(jb.err) + (size_t)b0 * jb.ldb * 4u;
        if (b0 + kTK <= p.B) {
            // a full pass: straight-line code, every request out before the first use
#pragma unroll
            for (int t = 0; t < kSteps; ++t) {
                gbytes ra = abase + (size_t)(4 * t) * jb.lda * 4u;
                gbytes rb = bbase + (size_t)(4 * t) * jb.ldb * 4u;
                asm volatile("" : "+s"(ra), "+s"(rb));
                a[t] = *(const __attribute__((address_space(1))) float*)(ra + la);
                b[t] = *(const __attribute__((address_space(1))) float*)(rb + lb);
            }
            return;
        }
#pragma unroll
        for (int t = 0; t < kSteps; ++t) {
            const unsigned int row = b0 + 4u * t;
            if (row + 4u <= p.B) {
                gbytes ra = abase + (size_t)(4 * t) * jb.lda * 4u;
                gbytes rb = bbase + (size_t)(4 * t) * jb.ldb * 4u;
                asm volatile("" : "+s"(ra), "+s"(rb));
                a[t] = *(const __attribute__((address_space(1))) float*)(ra + la);
                b[t] = *(const __attribute__((address_space(1))) float*)(rb + lb);
            } else if (row < p.B) {
                gbytes ra = abase + (size_t)(4 * t) * jb.lda * 4u;
                gbytes rb = bbase + (size_t)(4 * t) * jb.ldb * 4u;
                asm volatile("" : "+s"(ra), "+s"(rb));
                const float av = *(const __attribute__((address_space(1))) float*)(ra + la_c);
                const float bv = *(const __attribute__((address_space(1))) float*)(rb + lb_c);
                a[t] = row + lq < p.B ? av : 0.f;
                b[t] = row + lq < p.B ? bv : 0.f;
            } else {
                a[t] = 0.f;
                b[t] = 0.f;
            }
        }
    };
    load_pass(0);

    // bias corrections and the optimizer state of this lane's outputs
    const float c1 = p.ctr->c1, c2 = p.ctr->c2;
    const bool sync = p.wt && p.sync_every && p.ctr->adam_t % p.sync_every == 0;
    // (dueling head updated here: the lane of action nn holds the state of that action's
    // advantage weights instead; the state-value weight of row 4 lq + l16 of the quarter, and
    // of the bias row in lane 4, belongs to lanes l16 = 0 .. 4 of the left wavefronts)
    const bool fold = FOLD && j == p.fold_job;
    const unsigned int O = p.head_A + 1u;
    const bool colv = nn < p.head_A;
    const bool val_lane = fold && wc == 0 && (l16 < 4 || (l16 == 4 && do_bias));
    // (every load below is unconditional, from an index that is valid in every lane: a branch
    // here would make the wavefront wait for the operand loads in flight)
    float w_old[4], m_old[4], v_old[4];
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        const unsigned int k = fold ? p.head_off + (mm + v) * O + (colv ? 1u + nn : 0u)
                                    : jb.w_off + (mm + v) * jb.ldw + nn;
        w_old[v] = ldw(p.w, k);
        m_old[v] = ldw(p.m, k);
        v_old[v] = ldw(p.v, k);
    }
    const unsigned int hbias = p.head_off + jb.M * O;
    const unsigned int kb = fold ? hbias + (colv ? 1u + nn : 0u) : jb.b_off + nn;
    const float wb_old = ldw(p.w, kb), mb_old = ldw(p.m, kb), vb_old = ldw(p.v, kb);
    const unsigned int kval = !val_lane ? kb : l16 < 4 ? p.head_off + (mm + l16) * O : hbias;
    const float vw_old = ldw(p.w, kval), vm_old = ldw(p.m, kval), vv_old = ldw(p.v, kval);

    // the last workgroup of the launch that closes the step (never on a tile row with a bias)
    // also reduces the per-sample losses: fetch them now
    const bool loss_block = p.closes_step && block == p.n_tiles - 1;
    float loss_part = 0.f;
    if (loss_block && tid < 64)
        for (unsigned int i = tid; i < p.B; i += 64) loss_part += p.lossi[i];

    f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
    float bsum = 0.f;   // this lane's share of the column sum of Err (rows = lq mod 4)
    for (unsigned int b0 = 0; b0 < p.B; b0 += kTK) {
        if (b0 + kTK <= p.B) {
#pragma unroll
            for (int t = 0; t < kSteps; ++t) {
                acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a[t], b[t], acc, 0, 0, 0);
                if (bias_wave) bsum += b[t];
            }
        } else {
#pragma unroll
            for (int t = 0; t < kSteps; ++t) {
                if (b0 + 4u * t >= p.B) break;   // steps past the batch hold zeros
                acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a[t], b[t], acc, 0, 0, 0);
                if (bias_wave) bsum += b[t];
            }
        }
        if (b0 + kTK < p.B) load_pass(b0 + kTK);
    }
    if (bias_wave) {
        bsum += __shfl_xor(bsum, 16);
        bsum += __shfl_xor(bsum, 32);
    }

    // The optimizer state requested before the products has long arrived.  Naming every value
    // as an operand here makes the compiler wait for them now, before the first store: vmcnt
    // counts stores as well and retires in order, so a wait for one of these loads placed among
    // the stores below would also wait for the stores ahead of it to complete.
#pragma unroll
    for (int v = 0; v < 4; ++v) asm volatile("" ::"v"(w_old[v]), "v"(m_old[v]), "v"(v_old[v]));
    asm volatile("" ::"v"(wb_old), "v"(mb_old), "v"(vb_old), "v"(vw_old), "v"(vm_old), "v"(vv_old));
    const float r1 = 1.f / c1, r2 = 1.f / c2;
    if (fold) {
        // Dueling head (Q = V + A - mean A).  This lane holds dW[k][nn] of the plain layer for
        // hidden units k = mm .. mm+3 (entries 0..3) and, on the bias row, for k = H (entry 4).
        // The head's gradients are dV[k] = sum_a dW[k][a] and dA[k][a] = dW[k][a] - mean_a' dW[k][a'],
        // kept to the weights the head has (a gradient of zero where it has none: moments and
        // weight stay as they are); after their optimizer step the plain layer's row is rebuilt
        // as V[k] + A[k][a] - mean_a' A[k][a'].  A row's 32 columns sit in 16 lanes of each of the
        // two wavefronts of a tile row, so both sums take a lane reduction and a few words of LDS.
        __shared__ float hsum[2][2][17][2];   // [gradient / new weights][wr][row][wc]
        __shared__ float hval[2][17];         // new state-value weights [wr][row]
        const float inv_A = 1.f / (float)p.head_A;
        const unsigned int H = jb.M;
        const float x[5] = {acc[0], acc[1], acc[2], acc[3], bias_wave ? bsum : 0.f};
        float red[5];
#pragma unroll
        for (int i = 0; i < 5; ++i) red[i] = row16_sum(colv ? x[i] : 0.f);
        if (l16 == 0) {
#pragma unroll
            for (int i = 0; i < 4; ++i) hsum[0][wr][4u * lq + i][wc] = red[i];
            if (lq == 0) hsum[0][wr][16][wc] = red[4];
        }
        lds_barrier();   // (not __syncthreads: that would also wait for global stores in flight)
        float gsum[5];
#pragma unroll
        for (int i = 0; i < 5; ++i) {
            const unsigned int slot = i < 4 ? 4u * lq + i : 16u;
            gsum[i] = hsum[0][wr][slot][0] + hsum[0][wr][slot][1];
        }
        float a_new[5];   // this lane's new advantage weight (0 where the head has none)
#pragma unroll
        for (int i = 0; i < 5; ++i) a_new[i] = 0.f;
        if (colv) {
#pragma unroll
            for (int i = 0; i < 5; ++i) {
                if (i == 4 && !do_bias) continue;
                const unsigned int k = i < 4 ? mm + i : H;
                const bool a_on = head_connected(H, k, 1);
                const float wn = opt_apply(p, p.head_off + k * O + 1u + nn,
                                           a_on ? x[i] - gsum[i] * inv_A : 0.f,
                                           i < 4 ? w_old[i & 3] : wb_old, i < 4 ? m_old[i & 3] : mb_old,
                                           i < 4 ? v_old[i & 3] : vb_old, r1, r2, false, sync);
                a_new[i] = a_on ? wn : 0.f;
            }
        }
        if (val_lane) {
            const unsigned int k = l16 < 4 ? mm + l16 : H;
            const bool v_on = head_connected(H, k, 0);
            const unsigned int slot = l16 < 4 ? 4u * lq + l16 : 16u;
            const float gv = hsum[0][wr][slot][0] + hsum[0][wr][slot][1];
            const float wn = opt_apply(p, kval, v_on ? gv : 0.f, vw_old, vm_old, vv_old, r1, r2, false, sync);
            hval[wr][slot] = v_on ? wn : 0.f;
        }
#pragma unroll
        for (int i = 0; i < 5; ++i) red[i] = row16_sum(a_new[i]);
        if (l16 == 0) {
#pragma unroll
            for (int i = 0; i < 4; ++i) hsum[1][wr][4u * lq + i][wc] = red[i];
            if (lq == 0) hsum[1][wr][16][wc] = red[4];
        }
        lds_barrier();
        if (colv) {
#pragma unroll
            for (int i = 0; i < 5; ++i) {
                if (i == 4 && !do_bias) continue;
                const unsigned int slot = i < 4 ? 4u * lq + i : 16u;
                const unsigned int k = i < 4 ? mm + i : H;
                const float amean = (hsum[1][wr][slot][0] + hsum[1][wr][slot][1]) * inv_A;
                const float e = hval[wr][slot] + a_new[i] - amean;
                const unsigned int eff = (i < 4 ? jb.w_off + k * jb.ldw : jb.b_off) + nn;
                stw(p.w, eff, e);
                if (sync) stw(p.wt, eff, e);
            }
        }
    } else {
        const bool grad_only = j == p.grad_only_job;
        float w_new[4];
#pragma unroll
        for (int v = 0; v < 4; ++v)
            w_new[v] = opt_apply(p, jb.w_off + (mm + v) * jb.ldw + nn, acc[v], w_old[v], m_old[v],
                                 v_old[v], r1, r2, grad_only, sync);
        if (jb.wT)
            *reinterpret_cast<float4*>(jb.wT + (size_t)nn * jb.M + mm) =
                make_float4(w_new[0], w_new[1], w_new[2], w_new[3]);
        if (do_bias) opt_apply(p, jb.b_off + nn, bsum, wb_old, mb_old, vb_old, r1, r2, grad_only, sync);
    }
    if (loss_block && tid < 64) {
        const float s = wave_sum(loss_part);
        if (tid == 0) {
            p.ctr->loss = s / (float)p.B;
            p.ctr->step += 1;
        }
    }
}

template <bool FOLD>
__global__ __launch_bounds__(kThreads) void fused_weights_kernel(WArgs p) {
    touch_kernel_args<WArgs>();
    weights_tile<FOLD>(p, blockIdx.x);
}

// The launch of tiles of the fp32 step on MFMA, with two more kinds of workgroup in it:
//  - the first dz_blocks workgroups compute dZ1 = (dZ2 W2^T) masked by the first ReLU (16 x 16
//    per workgroup, K over its four wavefronts; dz_nx tiles per tile row).  The tiles of this
//    launch are then those that do not read dZ1 (the second layer's and the output layer's); the
//    first layer's follow in a launch of their own.  Product and tiles each fit the compute
//    units the other leaves idle, so the launch takes as long as the slower of the two alone.
//    The second layer's tiles update W2 in place, so the product takes W2 from a copy this
//    launch does not write (dz.B; made earlier in the step).
//  - after the tiles, next_blocks workgroups append, sample and gather for the NEXT train step
//    (inside a recorded run of steps): they touch nothing this step reads or writes (the next
//    step's batch goes to a buffer of its own), so the next step begins with its first layer.
template <bool FOLD>
__global__ __launch_bounds__(kThreads) void fused_weights_ahead_kernel(WArgs p, MmArgs dz, unsigned int dz_nx,
                                                                       unsigned int dz_blocks,
                                                                       AppendGatherArgs next,
                                                                       unsigned int next_blocks) {
    __shared__ float part[3][64][4];
    if (blockIdx.x < dz_blocks) {
        const unsigned int by = blockIdx.x / dz_nx;
        mm_f32_block<true, MM_MASK, true, 8>(dz, blockIdx.x - by * dz_nx, by, 0u, part);
        return;
    }
    const unsigned int block = blockIdx.x - dz_blocks;
    if (block >= p.n_tiles) {
        append_gather_block<4, kDrawUniform>(next, block - p.n_tiles, next_blocks);
        return;
    }
    weights_tile<FOLD>(p, block);
}

size_t row_kernel_lds(unsigned int Dp, unsigned int H, unsigned int Ap) {
    const size_t ldx = Dp + kPadK, ldh = H + kPadK, ldq = Ap + kPadK;
    return (8 * ldx + 8 * ldh * 2 + 8 * ldq + 4 * ldh + 16 * 8 * kChunk + (2 * H + Ap) + 16 + 4 +
            4 * kAheadWords + 4 * 64 + 4) *
           sizeof(float);
}

}  // namespace

bool fused_step_supported(const train_config& cfg, const replay* rp_) {
    if (cfg.param_dtype != RP_F32 || rp_->cfg.state_dtype != RP_F32 || rp_->cfg.layout != RP_PAIR)
        return false;
    // a lane owns one or four columns of a layer and holds its share of the weights in
    // registers: hidden width up to 256, states and action sets up to 64 wide
    if (cfg.hidden % 64 != 0 || cfg.hidden > 256 || cfg.state_dim > 64 || cfg.num_actions > 64)
        return false;
    if (cfg.hidden2 != 0 && cfg.hidden2 != cfg.hidden) return false;   // two layers of one width
    if (cfg.batch > 8192 || cfg.appends_per_step > 8192) return false;
    const unsigned int Dp = (unsigned int)align_up(cfg.state_dim, 32);
    const unsigned int Ap = (unsigned int)align_up(cfg.num_actions, 32);
    return row_kernel_lds(Dp, cfg.hidden, Ap) <= kRowLdsMax;
}

// The row kernel's dynamic LDS exceeds the default limit: announced once per process, at trainer
// creation (outside any stream capture).
hipError_t fused_init() {
    const void* kernels[] = {reinterpret_cast<const void*>(fused_rows_kernel<false, 8, 4>),
                             reinterpret_cast<const void*>(fused_rows_kernel<false, 16, 4>),
                             reinterpret_cast<const void*>(fused_rows_kernel<false, 8, 2>),
                             reinterpret_cast<const void*>(fused_rows_kernel<false, 16, 2>),
                             reinterpret_cast<const void*>(fused_rows_kernel<true, 8, 4>),
                             reinterpret_cast<const void*>(fused_rows_kernel<true, 16, 4>),
                             reinterpret_cast<const void*>(fused_rows_kernel<true, 8, 2>),
                             reinterpret_cast<const void*>(fused_rows_kernel<true, 16, 2>)};
    for (const void* k : kernels) {
        hipError_t e = hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kRowLdsMax);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// Experiences per workgroup of the row kernel: two while that still leaves compute units idle
// (every workgroup fetches all the weights, so more workgroups than that only add traffic); with
// a target network four per pair of workgroups.
unsigned int fused_rows_per_group(bool target_network, unsigned int B) {
    return B <= (target_network ? kSmallBatchSplit : kSmallBatch) ? 2u : kRows;
}

void* fused_rows_func(bool target_network, unsigned int Dp, unsigned int B) {
    const bool narrow = Dp <= 32;
    if (target_network) {
        if (fused_rows_per_group(true, B) == 2)
            return narrow ? reinterpret_cast<void*>(fused_rows_kernel<true, 8, 2>)
                          : reinterpret_cast<void*>(fused_rows_kernel<true, 16, 2>);
        return narrow ? reinterpret_cast<void*>(fused_rows_kernel<true, 8, 4>)
                      : reinterpret_cast<void*>(fused_rows_kernel<true, 16, 4>);
    }
    if (fused_rows_per_group(false, B) == 2)
        return narrow ? reinterpret_cast<void*>(fused_rows_kernel<false, 8, 2>)
                      : reinterpret_cast<void*>(fused_rows_kernel<false, 16, 2>);
    return narrow ? reinterpret_cast<void*>(fused_rows_kernel<false, 8, 4>)
                  : reinterpret_cast<void*>(fused_rows_kernel<false, 16, 4>);
}

hipError_t enqueue_fused_step(trainer* t, const Payload& src, const Payload* batch, hipStream_t st,
                              unsigned int* count) {
    replay* r = t->rp_;
    RowArgs& a = t->row_args;
    a.g = r->geom;
    a.seed = r->cfg.seed;
    a.n_append = batch ? 0u : t->cfg.appends_per_step;
    a.src = src;
    a.batch = batch ? *batch : Payload{nullptr, nullptr, nullptr, nullptr, nullptr};
    a.from_batch = batch ? 1u : 0u;
    {
        // state before this step, from the host mirrors (train_step has not advanced them yet)
        const unsigned long long cap = r->cfg.capacity, after = r->size + a.n_append;
        a.head = r->head;
        a.step = t->host_step;
        a.size_after = (unsigned int)(after > cap ? cap : after);
        a.next_size = (unsigned int)(after + a.n_append > cap ? cap : after + a.n_append);
        a.total_after = r->total + a.n_append;
        set_adam_step(a, t->host_adam_t + 1, t->cfg.beta1, t->cfg.beta2);
    }
    stamp_launch(t, a);
    a.ctr = t->ctr;
    a.w = t->w;
    a.wt = t->wt;
    a.w2t = t->w2t;
    a.B = t->B; a.D = t->cfg.state_dim; a.Dp = t->Dp; a.H = t->H; a.A = t->cfg.num_actions; a.Ap = t->Ap;
    a.oW1 = (unsigned int)t->oW1; a.ob1 = (unsigned int)t->ob1; a.oW2 = (unsigned int)t->oW2;
    a.ob2 = (unsigned int)t->ob2; a.oW3 = (unsigned int)t->oW3; a.ob3 = (unsigned int)t->ob3;
    a.gamma = t->cfg.gamma; a.beta1 = t->cfg.beta1; a.beta2 = t->cfg.beta2;
    a.loss_kind = t->cfg.loss;
    a.X = static_cast<float*>(t->X); a.H1 = static_cast<float*>(t->H1);
    a.H2 = static_cast<float*>(t->H2); a.Q = t->Q; a.y = t->y; a.delta = t->delta;
    a.lossi = t->lossi; a.dQ = t->dQ; a.dZ2 = static_cast<float*>(t->dZ2);
    a.dZ1 = static_cast<float*>(t->dZ1);
    a.act = t->act; a.rew = t->rew; a.term = t->term; a.idx = t->idx;
    // slots drawn a step ahead: when sampling without duplicates, for batches one workgroup covers
    // (the launch shape must not depend on the kind of step: graph launches reuse it)
    const bool ahead = r->cfg.sampling == RP_DISTINCT && t->B <= kRowThreads;
    a.pre = ahead ? t->pre : nullptr;
    a.pre_stride = 4u + t->B;
    const unsigned int per = fused_rows_per_group(t->wt != nullptr, t->B);
    // (with a target network: three workgroups for every four experiences)
    a.append_group = t->cfg.appends_per_step ? 1u : 0u;
    const unsigned int blocks = (t->B + per - 1) / per * (t->wt ? 3u : 1u) + a.append_group + (ahead ? 1u : 0u);
    hipError_t e = hipSuccess;
    void* kargs[] = {&a};
    e = hipLaunchKernel(fused_rows_func(t->wt != nullptr, t->Dp, t->B), dim3(blocks), dim3(kRowThreads), kargs,
                        row_kernel_lds(t->Dp, t->H, t->Ap), st);
    if (e != hipSuccess) return e;

    bool folded = false;
    e = enqueue_weights_update(t, st, &folded);
    if (e != hipSuccess) return e;
    unsigned int nh = 0;
    if (!folded) e = enqueue_head_update(t, st, &nh);
    if (count) *count = 2 + nh;
    return e;
}

namespace {

// What a recorded launch of fused_weights_ahead_kernel was given, apart from the next step's gather.
struct TilesRecorded {
    WArgs w;
    MmArgs dz;
    unsigned int dz_nx, dz_blocks;
};

// The tiles of the layers in `jobs` (bit j: job j; 0 = the second layer, 1 = the first, 2 = the output layer).
unsigned int set_weight_jobs(const trainer* t, unsigned int jobs, WArgs* w) {
    const unsigned int H = t->H, G = t->Hb;
    auto set = [&](int j, const float* act, unsigned int lda, const float* err, unsigned int ldb,
                   unsigned int M, unsigned int N, size_t w_off, size_t b_off, float* wT,
                   unsigned int begin) {
        WJob& jb = w->job[j];
        if (!(jobs >> j & 1u)) M = 0;
        jb.act = act; jb.lda = lda; jb.err = err; jb.ldb = ldb; jb.M = M; jb.N = N;
        jb.w_off = (unsigned int)w_off; jb.ldw = N; jb.b_off = (unsigned int)b_off; jb.wT = wT;
        jb.tiles_n = (N + kTN - 1) / kTN;
        jb.tile_begin = begin;
        return begin + jb.tiles_n * ((M + kTM - 1) / kTM);
    };
    unsigned int nt = 0;
    // (only the two-kernel step reads the transposed copy of W2)
    nt = set(0, static_cast<const float*>(t->H1), H, static_cast<const float*>(t->dZ2), G, H, G, t->oW2,
             t->ob2, t->fused ? t->w2t : nullptr, nt);
    nt = set(1, static_cast<const float*>(t->X), t->Dp, static_cast<const float*>(t->dZ1), H, t->Dp, H,
             t->oW1, t->ob1, nullptr, nt);
    nt = set(2, static_cast<const float*>(t->H2), G, t->dQ, t->Ap, G, t->Ap, t->oW3, t->ob3, nullptr, nt);
    return nt;
}

}  // namespace

// dz1 (fp32 step on MFMA): the product dZ1 to compute in the same launch as the tiles that do not
// read it; the first layer's tiles, which do, then follow in a second launch.
hipError_t enqueue_weights_update(trainer* t, hipStream_t st, bool* folded_head, const MmArgs* dz1,
                                  unsigned int* launches) {
    WArgs w;
    const unsigned int nt = set_weight_jobs(t, dz1 ? 0x5u : 0x7u, &w);
    w.B = t->B; w.n_tiles = nt;
    w.w = t->w; w.g = t->g; w.m = t->m; w.v = t->v;
    w.opt = t->cfg.opt; w.lr = t->cfg.lr; w.beta1 = t->cfg.beta1; w.beta2 = t->cfg.beta2;
    w.eps = t->cfg.eps; w.ctr = t->ctr; w.lossi = t->lossi;
    // the head of up to 32 actions (one tile column) is updated by job 2's own tiles
    const bool fold = t->dueling && t->Ap == kTN;
    w.grad_only_job = t->dueling && !fold ? 2u : ~0u;
    w.fold_job = fold ? 2u : ~0u;
    w.head_A = t->cfg.num_actions;
    w.head_off = (unsigned int)t->n_padded;
    w.wt = t->wt;
    w.sync_every = t->cfg.target_sync;
    w.closes_step = 1;
    if (launches) *launches = 1;
    if (t->rec_next || dz1) {
        TilesRecorded rec;
        memset(&rec, 0, sizeof(rec));
        rec.w = w;
        if (dz1) {
            rec.dz = *dz1;
            rec.dz_nx = dz1->N / 16u;
            rec.dz_blocks = rec.dz_nx * dz1->tiles_per_part;
        }
        AppendGatherArgs next;
        memset(&next, 0, sizeof(next));
        unsigned int nb = 0;
        size_t lds = 0;
        if (t->rec_next) {
            // (recording a run of steps: this launch also gathers the next step's batch; the argument
            // blocks are kept for the launches that replace the next step's part)
            if (!t->w_args_host[t->rec_parity]) t->w_args_host[t->rec_parity] = malloc(sizeof(TilesRecorded));
            if (!t->w_args_host[t->rec_parity]) return hipErrorOutOfMemory;
            memcpy(t->w_args_host[t->rec_parity], &rec, sizeof(TilesRecorded));
            next = *t->rec_next;
            append_gather_shape(next, &nb, &lds);
        }
        const dim3 grid(rec.dz_blocks + nt + nb);
        if (fold)
            hipLaunchKernelGGL(fused_weights_ahead_kernel<true>, grid, dim3(kThreads), lds, st, w, rec.dz,
                               rec.dz_nx, rec.dz_blocks, next, nb);
        else
            hipLaunchKernelGGL(fused_weights_ahead_kernel<false>, grid, dim3(kThreads), lds, st, w, rec.dz,
                               rec.dz_nx, rec.dz_blocks, next, nb);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        if (dz1) {
            WArgs w1 = w;
            w1.n_tiles = set_weight_jobs(t, 0x2u, &w1);
            w1.grad_only_job = ~0u;
            w1.fold_job = ~0u;
            w1.closes_step = 0;
            hipLaunchKernelGGL(fused_weights_kernel<false>, dim3(w1.n_tiles), dim3(kThreads), 0, st, w1);
            if (launches) *launches = 2;
        }
    } else if (fold) {
        hipLaunchKernelGGL(fused_weights_kernel<true>, dim3(nt), dim3(kThreads), 0, st, w);
    } else {
        hipLaunchKernelGGL(fused_weights_kernel<false>, dim3(nt), dim3(kThreads), 0, st, w);
    }
    if (folded_head) *folded_head = fold;
    return hipGetLastError();
}

void* weights_ahead_func(const trainer* t) {
    const bool fold = t->dueling && t->Ap == kTN;
    return fold ? reinterpret_cast<void*>(fused_weights_ahead_kernel<true>)
                : reinterpret_cast<void*>(fused_weights_ahead_kernel<false>);
}

hipError_t patch_weights_ahead_node(trainer* t, hipGraphExec_t exec, hipGraphNode_t node,
                                    const hipKernelNodeParams& recorded, unsigned int parity,
                                    const AppendGatherArgs& next) {
    TilesRecorded rec;
    memcpy(&rec, t->w_args_host[parity], sizeof(TilesRecorded));
    AppendGatherArgs nx = next;
    unsigned int nb = 0;
    size_t lds = 0;
    append_gather_shape(nx, &nb, &lds);
    void* kargs[] = {&rec.w, &rec.dz, &rec.dz_nx, &rec.dz_blocks, &nx, &nb};
    hipKernelNodeParams np = recorded;
    np.kernelParams = kargs;
    np.extra = nullptr;
    return hipGraphExecKernelNodeSetParams(exec, node, &np);
}

void free_weights_args(trainer* t) {
    for (auto& p : t->w_args_host) {
        free(p);
        p = nullptr;
    }
}

}  // namespace rp
