// Device code of the gather shared by the replay's own kernels and by the train steps that run the
// next step's append + gather inside another kernel's launch: a block of kGatherThreads threads
// numbered `block` out of `nblocks` does its share, wherever it runs.
//
// Paper: Methods (add, sample).
#pragma once
#include "common.hpp"
#include "philox.hpp"

namespace rp {

constexpr unsigned int kGatherThreads = 256;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// ---------------------------------------------------------------------------------------
// Append.  The ring state before the append comes as an argument (the host mirrors it exactly);
// one thread stores the state that follows.  Kernels that read the state run later in stream
// order.
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ void store_state_after(const RingGeom& g, const RingPos& pos,
                                                  unsigned long long n, unsigned int block = blockIdx.x) {
    if (block == 0 && threadIdx.x == 0) {
        unsigned long long h = pos.head + n;
        if (h >= g.capacity) h -= g.capacity;
        const unsigned long long sz = pos.size + n;
        g.state->head = h;
        g.state->size = sz > g.capacity ? g.capacity : sz;
        g.state->total = pos.total + n;
    }
}

// Word w of the packed PAIR row of payload experience `row`:
// [s | s' | pad to 4 | action | reward bits | terminal 0/1 | zero pad].
template <int ELEM>
__device__ __forceinline__ unsigned int payload_row_word(const RingGeom& g, const Payload& src,
                                                         unsigned long long row, unsigned int w) {
    const unsigned int o = w * 4u, sb = g.state_bytes;
    unsigned int val = 0;
    if (o < g.meta_off) {
        if (ELEM == 4) {
            const unsigned int col = w;
            val = col < g.state_dim
                      ? reinterpret_cast<const unsigned int*>(src.s)[row * g.state_dim + col]
                      : reinterpret_cast<const unsigned int*>(src.s_next)[row * g.state_dim + col -
                                                                          g.state_dim];
        } else if (ELEM == 2) {
#pragma unroll
            for (unsigned int h = 0; h < 2; ++h) {
                const unsigned int col = 2u * w + h;
                unsigned int half = 0;
                if (col < g.state_dim)
                    half = reinterpret_cast<const unsigned short*>(src.s)[row * g.state_dim + col];
                else if (col < 2u * g.state_dim)
                    half = reinterpret_cast<const unsigned short*>(src.s_next)[row * g.state_dim + col -
                                                                               g.state_dim];
                val |= half << (16 * h);
            }
        } else {
#pragma unroll
            for (unsigned int b = 0; b < 4; ++b) {
                const unsigned int ob = o + b;
                unsigned int byte = 0;
                if (ob < sb)
                    byte = src.s[row * sb + ob];
                else if (ob < 2 * sb)
                    byte = src.s_next[row * sb + ob - sb];
                val |= byte << (8 * b);
            }
        }
    } else if (o == g.meta_off) {
        val = (unsigned int)src.a[row];
    } else if (o == g.meta_off + 4) {
        val = __float_as_uint(src.r[row]);
    } else if (o == g.meta_off + 8) {
        val = src.term[row] ? 1u : 0u;
    }
    return val;
}

// float(b) / 255 for b in 0..255, correctly rounded: one multiply by the float nearest to
// 1/255 and one Newton correction through an exact FMA residual.  The result equals IEEE
// division for all 256 inputs (checked value by value in the tests).
__device__ __forceinline__ float unit_from_u8(unsigned int b) {
    constexpr float kInv255 = 0x1.010102p-8f;
    const float x = (float)b;
    const float q = x * kInv255;
    const float r = fmaf(-q, 255.0f, x);
    return fmaf(r, kInv255, q);
}

// ---------------------------------------------------------------------------------------
// Sample + gather + unpack, PAIR layout.  A block handles R = U * (256 >> lane_shift) batch
// rows.  The lanes that cooperate on a row (2^lane_shift of them, one 16-byte piece each for a
// 256-byte row) all draw the row's slot number themselves -- ten Philox rounds cost less than
// a trip through LDS and a barrier -- and fetch their pieces of U rows with all loads in
// flight at once; the rows go to LDS and then leave as contiguous, coalesced runs per output
// tensor.
// ---------------------------------------------------------------------------------------
// FRESH: `n_fresh` experiences from `fresh` are being appended at `head` by this same launch; a
// drawn slot among them is composed from those arrays instead of read from the ring.
// MODE: where a row's slot number comes from.  kDrawUniform: every lane of the row draws it
// (with replacement).  kDrawDistinct: without duplicates, drawn here by one lane per row.
// kDrawGiven: read from `drawn`, which an earlier kernel filled (see distinct_draw_kernel).
enum { kDrawUniform = 0, kDrawDistinct = 1, kDrawGiven = 2 };

// gather_pair_rows: batch rows i0 .. i0 + nrows - 1 (nrows <= R); with kDrawGiven, row i0 + rr
// takes slot number drawn[drawn_at + rr].
template <int ELEM, int U, int MODE, bool FRESH>
__device__ __forceinline__ void gather_pair_rows(const RingGeom& g, unsigned long long seed,
                                                 unsigned long long step, unsigned int size,
                                                 unsigned int lane_shift, const GatherOut& o,
                                                 const Payload& fresh, unsigned long long head,
                                                 unsigned long long n_fresh, const unsigned int* drawn,
                                                 unsigned int drawn_at, unsigned int i0, unsigned int nrows) {
    constexpr bool DISTINCT = MODE == kDrawDistinct;
    extern __shared__ uint4 smem[];
    unsigned int* idx_s = reinterpret_cast<unsigned int*>(smem);   // distinct mode: R slot numbers
    unsigned char* rows_s = reinterpret_cast<unsigned char*>(smem) + (DISTINCT ? 4 * U * kGatherThreads : 0);

    const unsigned int rows_per_pass = kGatherThreads >> lane_shift;

    {
        const unsigned int V = g.row_bytes >> 4;             // 16-byte vectors per row
        const unsigned int lanes = 1u << lane_shift;         // lanes per row (power of two)
        const unsigned int part0 = threadIdx.x & (lanes - 1u);
        const unsigned int rsub = threadIdx.x >> lane_shift;
        // A draw without duplicates takes some sixty dependent Philox blocks.  Where a row has
        // sixteen lanes and a thread one row, they make the draw as a team, four rounds at a
        // time (distinct_draw_team); otherwise one lane per row makes it.  The others pick it
        // up from LDS.
        if constexpr (DISTINCT) {
            if (U == 1 && lane_shift == 4) {
                __shared__ unsigned int keys[kDistinctTableWords];
                const unsigned int rounds = distinct_rounds(size);
                if (threadIdx.x < 64u) {
                    if (threadIdx.x < kDistinctTableWords - 64u) keys[64u + threadIdx.x] = 0u;
                    distinct_round_keys(seed, step, size, rounds, threadIdx.x, keys);
                }
                __syncthreads();
                const unsigned int u = distinct_draw_team<4>(seed, step, i0 + (rsub < nrows ? rsub : 0u), size,
                                                             rounds, keys, threadIdx.x & 63u);
                if (part0 == 0) idx_s[rsub] = u;
            } else {
                for (unsigned int rr = threadIdx.x; rr < nrows; rr += kGatherThreads)
                    idx_s[rr] = distinct_draw(seed, step, i0 + rr, size);
            }
            __syncthreads();
        }
        const unsigned char* src[U];
        unsigned long long fresh_row[U];
        bool is_fresh[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            unsigned int rr = rsub + u * rows_per_pass;
            rr = rr < nrows ? rr : 0u;   // a row past the end re-reads row 0; not stored
            const unsigned int p = MODE == kDrawGiven ? drawn[drawn_at + rr]
                                   : DISTINCT         ? idx_s[rr]
                                                      : uniform_draw(seed, step, i0 + rr, size);
            src[u] = g.rows + (unsigned long long)p * g.row_bytes;
            unsigned long long off = (unsigned long long)p + g.capacity - head;
            if (off >= g.capacity) off -= g.capacity;
            fresh_row[u] = off;
            is_fresh[u] = FRESH && off < n_fresh;
            if (o.out_idx && part0 == 0 && rsub + u * rows_per_pass < nrows) o.out_idx[i0 + rr] = p;
        }
        for (unsigned int part = part0; part < V; part += lanes) {
            // (a native vector type: an array of HIP's uint4 struct would live in scratch memory)
            u32x4 val[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (FRESH && is_fresh[u]) {
#pragma unroll
                    for (unsigned int j = 0; j < 4; ++j)
                        val[u][j] = payload_row_word<ELEM>(g, fresh, fresh_row[u], 4u * part + j);
                } else {
                    val[u] = reinterpret_cast<const u32x4*>(src[u])[part];
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const unsigned int rr = rsub + u * rows_per_pass;
                if (rr < nrows)
                    reinterpret_cast<u32x4*>(rows_s + (size_t)rr * g.row_bytes)[part] = val[u];
            }
        }
    }
    __syncthreads();

    // unpack: 32 lanes walk the columns of one row, 8 rows per pass; consecutive rows are
    // adjacent in the output, so a wavefront writes one contiguous run
    const unsigned int D = g.state_dim;
    for (unsigned int row = threadIdx.x >> 5; row < nrows; row += kGatherThreads >> 5) {
        const unsigned char* base = rows_s + (size_t)row * g.row_bytes;
        const size_t at = (size_t)(i0 + row) * o.out_ld;
        for (unsigned int col = threadIdx.x & 31u; col < D; col += 32) {
            if (ELEM == 4) {
                const unsigned int* w = reinterpret_cast<const unsigned int*>(base);
                if (o.out_s) static_cast<unsigned int*>(o.out_s)[at + col] = w[col];
                if (o.out_s_next) static_cast<unsigned int*>(o.out_s_next)[at + col] = w[D + col];
                if (o.out_s_t) static_cast<unsigned int*>(o.out_s_t)[(size_t)col * o.out_t_ld + i0 + row] = w[col];
            } else if (ELEM == 2) {
                const unsigned short* h = reinterpret_cast<const unsigned short*>(base);
                if (o.out_s) static_cast<unsigned short*>(o.out_s)[at + col] = h[col];
                if (o.out_s_next) static_cast<unsigned short*>(o.out_s_next)[at + col] = h[D + col];
                if (o.out_s_t) static_cast<unsigned short*>(o.out_s_t)[(size_t)col * o.out_t_ld + i0 + row] = h[col];
            } else {
                if (o.out_s) static_cast<float*>(o.out_s)[at + col] = unit_from_u8(base[col]);
                if (o.out_s_next) static_cast<float*>(o.out_s_next)[at + col] = unit_from_u8(base[D + col]);
            }
        }
    }
    for (unsigned int row = threadIdx.x; row < nrows; row += kGatherThreads) {
        const unsigned int i = i0 + row;
        const unsigned int* meta =
            reinterpret_cast<const unsigned int*>(rows_s + (size_t)row * g.row_bytes + g.meta_off);
        if (o.out_a) o.out_a[i] = (int)meta[0];
        if (o.out_r) o.out_r[i] = __uint_as_float(meta[1]);
        if (o.out_term) o.out_term[i] = (unsigned char)meta[2];
    }
}

template <int ELEM, int U, int MODE, bool FRESH>
__device__ __forceinline__ void gather_pair_block(const RingGeom& g, unsigned long long seed,
                                                  unsigned long long step, unsigned int size,
                                                  unsigned int batch, unsigned int lane_shift,
                                                  const GatherOut& o, const Payload& fresh,
                                                  unsigned long long head, unsigned long long n_fresh,
                                                  const unsigned int* __restrict__ drawn = nullptr,
                                                  unsigned int block = blockIdx.x) {
    const unsigned int R = U * (kGatherThreads >> lane_shift);
    const unsigned int i0 = block * R;
    gather_pair_rows<ELEM, U, MODE, FRESH>(g, seed, step, size, lane_shift, o, fresh, head, n_fresh, drawn, i0,
                                           i0, min(R, batch - i0));
}


// Append, then sample and gather, as block `block` of `nblocks` (the first kernel of the train
// steps on MFMA, or extra blocks of another kernel's launch).  The ring state before the append
// comes by value.  The blocks share the new rows out among themselves and send them to the ring
// first; nobody reads those slots from the ring in this launch (see FRESH above), so the order of
// the two halves within the launch does not matter.  Needs append_gather_shape's dynamic LDS.
template <int ELEM, int MODE>
__device__ __forceinline__ void append_gather_block(const AppendGatherArgs& p, unsigned int block,
                                                    unsigned int nblocks) {
    const RingGeom& g = p.g;
    store_state_after(g, p.pos, p.n, block);
    const unsigned int words = g.row_bytes >> 2;
    for (unsigned long long row = block; row < p.n; row += nblocks) {
        unsigned long long slot = p.pos.head + row;
        if (slot >= g.capacity) slot -= g.capacity;
        for (unsigned int w = threadIdx.x; w < words; w += kGatherThreads)
            reinterpret_cast<unsigned int*>(g.rows + slot * g.row_bytes)[w] =
                payload_row_word<ELEM>(g, p.src, row, w);
    }
    const unsigned long long sz = p.pos.size + p.n;
    const unsigned int size = (unsigned int)(sz > g.capacity ? g.capacity : sz);
    gather_pair_block<ELEM, 1, MODE, true>(g, p.seed, p.step_ptr ? *p.step_ptr : p.step_value, size, p.batch,
                                           p.lane_shift, p.out, p.src, p.pos.head, p.n, nullptr, block);
}

}  // namespace rp
