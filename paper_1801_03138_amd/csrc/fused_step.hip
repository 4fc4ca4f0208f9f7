// Two-kernel train step for small fp32 networks, where the step is bound by launch latency
// and by dependent phases rather than by arithmetic.
//
// Everything that concerns one sampled experience is independent of the other rows of the
// batch: its slot draw, its gather, the forward pass on s and s', the TD target, and the
// backward pass down to the pre-activation gradients.  Kernel 1 does all of that for four
// experiences per workgroup, keeping activations in LDS and streaming the weights through
// 4x4x1 fp32 MFMA (four rows per instruction, so a four-row tile is not padded).  It also
// appends the step's new experiences.  Only the weight gradients reduce over the batch:
// kernel 2 forms them tile by tile and applies the optimizer to each tile as soon as it is
// complete, so gradients never make a round trip through HBM before the update.
//
// Paper: Integration with Reinforcement Learning Algorithm (train step with no host inputs),
// Deep Q-Network Model (update equation), Methods (add, sample).
#include "philox.hpp"
#include "trainer.hpp"

namespace rp {
namespace {

constexpr unsigned int kThreads = kTrainThreads;
constexpr unsigned int kRows = 4;          // experiences per workgroup of the row kernel
constexpr unsigned int kChunk = 256;       // output columns one wavefront covers per pass
constexpr unsigned int kPadK = 4;          // LDS row padding (floats) against bank conflicts

typedef float f32x4 __attribute__((ext_vector_type(4)));

struct RowArgs {
    RingGeom g;
    unsigned long long seed;
    unsigned int n_append;
    const unsigned char* st_s;
    const unsigned char* st_s_next;
    const int* st_a;
    const float* st_r;
    const unsigned char* st_term;
    TrainCounters* ctr;
    const float* w;       // padded parameters
    const float* w2t;     // W2 transposed
    unsigned int B, D, Dp, H, A, Ap;
    unsigned int oW1, ob1, oW2, ob2, oW3, ob3;
    float gamma, beta1, beta2;
    unsigned int loss_kind;
    float *X, *H1, *H2, *Q, *y, *delta, *lossi, *dQ, *dZ2, *dZ1;
    int* act;
    float* rew;
    unsigned char* term;
    unsigned int* idx;
};

// One 32-bit word of the packed row of a new experience, taken from the staging arrays.
__device__ __forceinline__ unsigned int staged_word(const RowArgs& p, unsigned long long k,
                                                    unsigned int w) {
    const unsigned int D = p.D;
    if (w < D) return reinterpret_cast<const unsigned int*>(p.st_s)[k * D + w];
    if (w < 2 * D) return reinterpret_cast<const unsigned int*>(p.st_s_next)[k * D + w - D];
    if (w == 2 * D) return (unsigned int)p.st_a[k];
    if (w == 2 * D + 1) return __float_as_uint(p.st_r[k]);
    if (w == 2 * D + 2) return p.st_term[k] ? 1u : 0u;
    return 0u;
}

// part[wave][row][col] = sum over this wavefront's quarter of K of act[row][k] * W[k][col]
// for MG*4 rows and the 256 columns of `chunk`.  act: LDS, row pitch ldk floats.  W: global,
// row-major [K x N], N a multiple of 4, K a multiple of 16.  Each lane loads a float4 of
// four adjacent columns per k (1 KB per wavefront, fully coalesced) and feeds one column
// group per MFMA; the activations come in as the broadcast A operand.
template <int MG>
__device__ __forceinline__ void mm_rows(const float* act, unsigned int ldk, unsigned int K,
                                        const float* __restrict__ W, unsigned int N,
                                        unsigned int chunk, float* part) {
    const unsigned int lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    const unsigned int col = chunk * kChunk + 4u * lane;
    const bool active = col < N;
    const unsigned int Kq = K >> 2;
    const unsigned int kbeg = wave * Kq, kend = kbeg + Kq;
    const float* wp = W + col;
    const float* ap = act + (lane & 3u) * ldk;

    f32x4 acc[MG][4];
#pragma unroll
    for (int mg = 0; mg < MG; ++mg)
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) acc[mg][gq] = f32x4{0.f, 0.f, 0.f, 0.f};

    constexpr int U = 16;  // k rows per pipeline stage
    f32x4 cur[U], nxt[U];
    auto load_stage = [&](f32x4* dst, unsigned int k0) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const unsigned int k = k0 + u;
            dst[u] = (active && k < kend)
                         ? *reinterpret_cast<const f32x4*>(wp + (size_t)k * N)
                         : f32x4{0.f, 0.f, 0.f, 0.f};
        }
    };
    load_stage(cur, kbeg);
    for (unsigned int k0 = kbeg; k0 < kend; k0 += U) {
        if (k0 + U < kend) load_stage(nxt, k0 + U);
#pragma unroll
        for (int u4 = 0; u4 < U; u4 += 4) {
            if (k0 + u4 < kend) {  // Kq is a multiple of 4, so a group of four is all in or all out
#pragma unroll
                for (int mg = 0; mg < MG; ++mg) {
                    const f32x4 a = *reinterpret_cast<const f32x4*>(ap + (size_t)mg * 4 * ldk + k0 + u4);
#pragma unroll
                    for (int u = 0; u < 4; ++u)
#pragma unroll
                        for (int gq = 0; gq < 4; ++gq)
                            acc[mg][gq] = __builtin_amdgcn_mfma_f32_4x4x1f32(
                                a[u], cur[u4 + u][gq], acc[mg][gq], 0, 0, 0);
                }
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) cur[u] = nxt[u];
    }
    // lane holds, for column group gq, rows v = 0..3 of column 4*lane + gq
#pragma unroll
    for (int mg = 0; mg < MG; ++mg)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            float* dst = part + ((size_t)(wave * (MG * 4) + mg * 4 + v)) * kChunk + 4u * lane;
            *reinterpret_cast<f32x4*>(dst) =
                f32x4{acc[mg][0][v], acc[mg][1][v], acc[mg][2][v], acc[mg][3][v]};
        }
}

// sum of the four wavefronts' partial products for (row, col of the current chunk)
template <int MG>
__device__ __forceinline__ float part_sum(const float* part, unsigned int row, unsigned int c) {
    float v = part[(size_t)(0 * MG * 4 + row) * kChunk + c];
    v += part[(size_t)(1 * MG * 4 + row) * kChunk + c];
    v += part[(size_t)(2 * MG * 4 + row) * kChunk + c];
    v += part[(size_t)(3 * MG * 4 + row) * kChunk + c];
    return v;
}

// out[row][col] = relu?(in[row][:] . W[:, col] + bias[col]) for the 8 rows (4 of s, 4 of s').
// Rows 0..3 are also written to the global activation array `glob` (row pitch N) when given.
__device__ __forceinline__ void dense_rows8(const float* in, unsigned int ldk, unsigned int K,
                                            const float* __restrict__ W,
                                            const float* __restrict__ bias, unsigned int N,
                                            bool relu, float* out, unsigned int ldo, float* part,
                                            float* __restrict__ glob, unsigned int i0,
                                            unsigned int nrows) {
    for (unsigned int chunk = 0; chunk * kChunk < N; ++chunk) {
        mm_rows<2>(in, ldk, K, W, N, chunk, part);
        __syncthreads();
        const unsigned int ncol = min(kChunk, N - chunk * kChunk);
        for (unsigned int e = threadIdx.x; e < 8 * ncol; e += kThreads) {
            const unsigned int row = e / ncol, c = e - row * ncol, col = chunk * kChunk + c;
            float v = part_sum<2>(part, row, c) + bias[col];
            if (relu) v = v > 0.f ? v : 0.f;
            out[(size_t)row * ldo + col] = v;
            if (glob && row < nrows) glob[(size_t)(i0 + row) * N + col] = v;
        }
        __syncthreads();
    }
}

__global__ __launch_bounds__(kThreads) void fused_rows_kernel(RowArgs p) {
    extern __shared__ float lds[];
    const unsigned int tid = threadIdx.x;
    const unsigned int D = p.D, Dp = p.Dp, H = p.H, A = p.A, Ap = p.Ap;
    const unsigned int ldx = Dp + kPadK, ldh = H + kPadK, ldq = Ap + kPadK;
    float* Xs = lds;                      // [8][ldx]  rows 0..3 = s, 4..7 = s'
    float* H1s = Xs + 8 * ldx;            // [8][ldh]
    float* H2s = H1s + 8 * ldh;           // [8][ldh]
    float* Qs = H2s + 8 * ldh;            // [8][ldq]
    float* dZs = Qs + 8 * ldq;            // [4][ldh]
    float* part = dZs + 4 * ldh;          // [4 waves][8][256]
    unsigned int* meta = reinterpret_cast<unsigned int*>(part + 4 * 8 * kChunk);  // [4][4]
    float* gs = reinterpret_cast<float*>(meta + 16);                              // [4]

    // ring and trainer state as they stand before this step's append
    const unsigned long long cap = p.g.capacity;
    const unsigned long long head = p.g.state->head;
    const unsigned long long size0 = p.g.state->size;
    const unsigned long long step = p.ctr->step;
    const unsigned long long n = p.n_append;
    const unsigned int size = (unsigned int)(size0 + n > cap ? cap : size0 + n);
    const unsigned int i0 = blockIdx.x * kRows;
    const unsigned int nrows = min(kRows, p.B - i0);

    if (blockIdx.x == 0 && tid == 0) {
        const unsigned long long t = p.ctr->adam_t + 1;
        p.ctr->adam_t = t;
        p.ctr->c1 = (float)(1.0 - pow((double)p.beta1, (double)t));
        p.ctr->c2 = (float)(1.0 - pow((double)p.beta2, (double)t));
    }

    for (unsigned int e = tid; e < 8 * ldx; e += kThreads) Xs[e] = 0.f;
    if (tid < 16) meta[tid] = 0;
    __syncthreads();

    // sample and gather: one 32-bit word per thread.  A drawn slot that this step's append is
    // about to overwrite is read from the staging arrays, which hold its new content.
    const unsigned int words = 2 * D + 3;
    for (unsigned int e = tid; e < nrows * words; e += kThreads) {
        const unsigned int r = e / words, w = e - r * words;
        const unsigned int i = i0 + r;
        const unsigned int slot = uniform_draw(p.seed, step, i, size);
        unsigned long long off = (unsigned long long)slot + cap - head;
        if (off >= cap) off -= cap;
        const unsigned int val =
            off < n ? staged_word(p, off, w)
                    : reinterpret_cast<const unsigned int*>(p.g.rows + (unsigned long long)slot * p.g.row_bytes)[w];
        if (w < D) {
            Xs[r * ldx + w] = __uint_as_float(val);
            p.X[(size_t)i * Dp + w] = __uint_as_float(val);
        } else if (w < 2 * D) {
            Xs[(4 + r) * ldx + w - D] = __uint_as_float(val);
        } else {
            meta[r * 4 + (w - 2 * D)] = val;
            if (w == 2 * D) {
                p.act[i] = (int)val;
                p.idx[i] = slot;
            } else if (w == 2 * D + 1) {
                p.rew[i] = __uint_as_float(val);
            } else {
                p.term[i] = (unsigned char)val;
            }
        }
    }
    __syncthreads();

    // forward on the eight rows
    const float* W1 = p.w + p.oW1;
    const float* W2 = p.w + p.oW2;
    const float* W3 = p.w + p.oW3;
    dense_rows8(Xs, ldx, Dp, W1, p.w + p.ob1, H, true, H1s, ldh, part, p.H1, i0, nrows);
    dense_rows8(H1s, ldh, H, W2, p.w + p.ob2, H, true, H2s, ldh, part, p.H2, i0, nrows);
    dense_rows8(H2s, ldh, H, W3, p.w + p.ob3, Ap, false, Qs, ldq, part, nullptr, i0, nrows);

    // Q values out (rows i and B+i of the [2B x Ap] array), then TD target, loss term, dL/dQ
    for (unsigned int e = tid; e < 8 * Ap; e += kThreads) {
        const unsigned int row = e / Ap, c = e - row * Ap, r = row & 3u;
        if (r < nrows)
            p.Q[((size_t)(row < 4 ? 0 : p.B) + i0 + r) * Ap + c] = Qs[row * ldq + c];
    }
    if (tid < nrows) {
        const unsigned int r = tid, i = i0 + r;
        float best = -INFINITY;
        for (unsigned int k = 0; k < A; ++k) best = fmaxf(best, Qs[(4 + r) * ldq + k]);
        unsigned int ai = meta[r * 4 + 0];
        if (ai >= A) ai = A - 1;  // an out-of-range action must not turn into a wild address
        meta[r * 4 + 3] = ai;
        const float q = Qs[r * ldq + ai];
        const float y = __uint_as_float(meta[r * 4 + 1]) + (meta[r * 4 + 2] ? 0.f : p.gamma * best);
        const float d = y - q;
        float li, slope;
        if (p.loss_kind == RP_MSE || fabsf(d) <= 1.f) {
            li = 0.5f * d * d;
            slope = d;
        } else {
            li = fabsf(d) - 0.5f;
            slope = d > 0.f ? 1.f : -1.f;
        }
        const float gr = -slope / (float)p.B;
        gs[r] = gr;
        p.y[i] = y;
        p.delta[i] = d;
        p.lossi[i] = li;
    }
    __syncthreads();
    for (unsigned int e = tid; e < nrows * Ap; e += kThreads) {
        const unsigned int r = e / Ap, c = e - r * Ap;
        p.dQ[(size_t)(i0 + r) * Ap + c] = (c == meta[r * 4 + 3]) ? gs[r] : 0.f;
    }

    // dZ2[r][k] = dQ[r][a_r] * W3[k][a_r] * 1[H2[r][k] > 0]
    for (unsigned int e = tid; e < 4 * H; e += kThreads) {
        const unsigned int r = e / H, k = e - r * H;
        float v = 0.f;
        if (r < nrows && H2s[r * ldh + k] > 0.f) v = gs[r] * W3[(size_t)k * Ap + meta[r * 4 + 3]];
        dZs[r * ldh + k] = v;
        if (r < nrows) p.dZ2[(size_t)(i0 + r) * H + k] = v;
    }
    __syncthreads();

    // dZ1 = (dZ2 W2^T) masked by the first ReLU, through the transposed copy of W2
    for (unsigned int chunk = 0; chunk * kChunk < H; ++chunk) {
        mm_rows<1>(dZs, ldh, H, p.w2t, H, chunk, part);
        __syncthreads();
        const unsigned int ncol = min(kChunk, H - chunk * kChunk);
        for (unsigned int e = tid; e < nrows * ncol; e += kThreads) {
            const unsigned int r = e / ncol, c = e - r * ncol, col = chunk * kChunk + c;
            float v = part_sum<1>(part, r, c);
            if (!(H1s[r * ldh + col] > 0.f)) v = 0.f;
            p.dZ1[(size_t)(i0 + r) * H + col] = v;
        }
        __syncthreads();
    }

    // the last workgroup writes the new experiences into the ring
    if (blockIdx.x == gridDim.x - 1 && n) {
        const unsigned int rw = p.g.row_bytes >> 2;
        for (unsigned long long e = tid; e < n * rw; e += kThreads) {
            const unsigned long long k = e / rw;
            const unsigned int w = (unsigned int)(e - k * rw);
            unsigned long long slot = head + k;
            if (slot >= cap) slot -= cap;
            reinterpret_cast<unsigned int*>(p.g.rows + slot * p.g.row_bytes)[w] = staged_word(p, k, w);
        }
    }
    // every workgroup read the ring state before this point; the last one to arrive advances it
    __threadfence();
    __syncthreads();
    if (tid == 0) {
        const unsigned int done = atomicAdd(&p.g.state->blocks_done, 1u);
        if (done == gridDim.x - 1) {
            unsigned long long h = head + n;
            if (h >= cap) h -= cap;
            p.g.state->head = h;
            p.g.state->size = size;
            p.g.state->total += n;
            p.g.state->blocks_done = 0;
            __threadfence();
        }
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
};

constexpr unsigned int kTM = 32, kTN = 64, kTK = 64;

__device__ __forceinline__ float opt_update(const WArgs& p, unsigned int k, float gk, float c1,
                                            float c2) {
    float wk = p.w[k];
    p.g[k] = gk;
    if (p.opt == RP_SGD) {
        wk -= p.lr * gk;
    } else {
        const float mk = p.beta1 * p.m[k] + (1.f - p.beta1) * gk;
        const float vk = p.beta2 * p.v[k] + (1.f - p.beta2) * gk * gk;
        p.m[k] = mk;
        p.v[k] = vk;
        wk -= p.lr * (mk / c1) / (sqrtf(vk / c2) + p.eps);
    }
    p.w[k] = wk;
    return wk;
}

__global__ __launch_bounds__(kThreads) void fused_weights_kernel(WArgs p) {
    __shared__ float As[kTK][kTM + 1];
    __shared__ float Bs[kTK][kTN + 4];
    const unsigned int tid = threadIdx.x;
    unsigned int j = 0;
    if (blockIdx.x >= p.job[1].tile_begin) j = 1;
    if (blockIdx.x >= p.job[2].tile_begin) j = 2;
    const WJob& jb = p.job[j];
    const unsigned int tile = blockIdx.x - jb.tile_begin;
    const unsigned int m0 = (tile / jb.tiles_n) * kTM, n0 = (tile % jb.tiles_n) * kTN;
    const unsigned int ty = tid >> 4, tx = tid & 15u;  // rows 2*ty.., columns 4*tx..
    float acc[2][4] = {};
    float bsum[4] = {};
    const bool do_bias = m0 == 0 && ty == 0;

    for (unsigned int b0 = 0; b0 < p.B; b0 += kTK) {
        for (unsigned int e = tid; e < kTK * kTM; e += kThreads) {
            const unsigned int i = e / kTM, c = e % kTM;
            const unsigned int bi = b0 + i, m = m0 + c;
            As[i][c] = (bi < p.B && m < jb.M) ? jb.act[(size_t)bi * jb.lda + m] : 0.f;
        }
        for (unsigned int e = tid; e < kTK * kTN; e += kThreads) {
            const unsigned int i = e / kTN, c = e % kTN;
            const unsigned int bi = b0 + i, nn = n0 + c;
            Bs[i][c] = (bi < p.B && nn < jb.N) ? jb.err[(size_t)bi * jb.ldb + nn] : 0.f;
        }
        __syncthreads();
#pragma unroll 8
        for (unsigned int i = 0; i < kTK; ++i) {
            const float a0 = As[i][2 * ty], a1 = As[i][2 * ty + 1];
            const float4 b = *reinterpret_cast<const float4*>(&Bs[i][4 * tx]);
            acc[0][0] = fmaf(a0, b.x, acc[0][0]); acc[0][1] = fmaf(a0, b.y, acc[0][1]);
            acc[0][2] = fmaf(a0, b.z, acc[0][2]); acc[0][3] = fmaf(a0, b.w, acc[0][3]);
            acc[1][0] = fmaf(a1, b.x, acc[1][0]); acc[1][1] = fmaf(a1, b.y, acc[1][1]);
            acc[1][2] = fmaf(a1, b.z, acc[1][2]); acc[1][3] = fmaf(a1, b.w, acc[1][3]);
            if (do_bias) {
                bsum[0] += b.x; bsum[1] += b.y; bsum[2] += b.z; bsum[3] += b.w;
            }
        }
        __syncthreads();
    }

    const float c1 = p.ctr->c1, c2 = p.ctr->c2;
#pragma unroll
    for (int r = 0; r < 2; ++r) {
        const unsigned int m = m0 + 2 * ty + r;
        if (m >= jb.M) continue;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const unsigned int nn = n0 + 4 * tx + c;
            if (nn >= jb.N) continue;
            const float wk = opt_update(p, jb.w_off + m * jb.ldw + nn, acc[r][c], c1, c2);
            if (jb.wT) jb.wT[(size_t)nn * jb.M + m] = wk;
        }
    }
    if (do_bias) {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const unsigned int nn = n0 + 4 * tx + c;
            if (nn < jb.N) opt_update(p, jb.b_off + nn, bsum[c], c1, c2);
        }
    }
    if (blockIdx.x == 0 && tid < 64) {
        float s = 0.f;
        for (unsigned int i = tid; i < p.B; i += 64) s += p.lossi[i];
        s = wave_sum(s);
        if (tid == 0) {
            p.ctr->loss = s / (float)p.B;
            p.ctr->step += 1;
        }
    }
}

size_t row_kernel_lds(unsigned int Dp, unsigned int H, unsigned int Ap) {
    const size_t ldx = Dp + kPadK, ldh = H + kPadK, ldq = Ap + kPadK;
    return (8 * ldx + 8 * ldh * 2 + 8 * ldq + 4 * ldh + 4 * 8 * kChunk + 16 + 4) * sizeof(float);
}

}  // namespace

bool fused_step_supported(const train_config& cfg, const replay* rp_) {
    if (cfg.param_dtype != RP_F32 || rp_->cfg.state_dtype != RP_F32 || rp_->cfg.layout != RP_PAIR)
        return false;
    if (cfg.hidden % 64 != 0 || cfg.hidden > 512 || cfg.state_dim > 224 || cfg.num_actions > 224)
        return false;
    if (cfg.batch > 8192 || cfg.appends_per_step > 8192) return false;
    const unsigned int Dp = (unsigned int)align_up(cfg.state_dim, 32);
    const unsigned int Ap = (unsigned int)align_up(cfg.num_actions, 32);
    return row_kernel_lds(Dp, cfg.hidden, Ap) <= 64 * 1024;
}

hipError_t enqueue_fused_step(trainer* t, hipStream_t st, unsigned int* count) {
    replay* r = t->rp_;
    RowArgs a;
    a.g = r->geom;
    a.seed = r->cfg.seed;
    a.n_append = t->cfg.appends_per_step;
    a.st_s = r->stage_s;
    a.st_s_next = r->stage_s_next;
    a.st_a = r->stage_a;
    a.st_r = r->stage_r;
    a.st_term = r->stage_term;
    a.ctr = t->ctr;
    a.w = t->w;
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
    const unsigned int blocks = (t->B + kRows - 1) / kRows;
    hipLaunchKernelGGL(fused_rows_kernel, dim3(blocks), dim3(kThreads),
                       row_kernel_lds(t->Dp, t->H, t->Ap), st, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;

    WArgs w;
    const unsigned int H = t->H;
    auto set = [&](int j, const float* act, unsigned int lda, const float* err, unsigned int ldb,
                   unsigned int M, unsigned int N, size_t w_off, size_t b_off, float* wT,
                   unsigned int begin) {
        WJob& jb = w.job[j];
        jb.act = act; jb.lda = lda; jb.err = err; jb.ldb = ldb; jb.M = M; jb.N = N;
        jb.w_off = (unsigned int)w_off; jb.ldw = N; jb.b_off = (unsigned int)b_off; jb.wT = wT;
        jb.tiles_n = (N + kTN - 1) / kTN;
        jb.tile_begin = begin;
        return begin + jb.tiles_n * ((M + kTM - 1) / kTM);
    };
    unsigned int nt = 0;
    nt = set(0, a.H1, H, a.dZ2, H, H, H, t->oW2, t->ob2, t->w2t, nt);
    nt = set(1, a.X, t->Dp, a.dZ1, H, t->Dp, H, t->oW1, t->ob1, nullptr, nt);
    nt = set(2, a.H2, H, t->dQ, t->Ap, H, t->Ap, t->oW3, t->ob3, nullptr, nt);
    w.B = t->B; w.n_tiles = nt;
    w.w = t->w; w.g = t->g; w.m = t->m; w.v = t->v;
    w.opt = t->cfg.opt; w.lr = t->cfg.lr; w.beta1 = t->cfg.beta1; w.beta2 = t->cfg.beta2;
    w.eps = t->cfg.eps; w.ctr = t->ctr; w.lossi = t->lossi;
    hipLaunchKernelGGL(fused_weights_kernel, dim3(nt), dim3(kThreads), 0, st, w);
    if (count) *count = 2;
    return hipGetLastError();
}

}  // namespace rp
