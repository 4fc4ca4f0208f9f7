// The Q-learning train step on a device-resident replay: sample + gather, MLP forward on
// s and s', TD target / selection / loss, backward, optimizer, replayed as one HIP graph.
//
// Paper: Integration with Reinforcement Learning Algorithm (the step takes no inputs from
// the host; Q(s,a) is entry i*A + a_i of the flattened network output) and Deep Q-Network
// Model (the update equation).
#include <algorithm>
#include <cmath>
#include <vector>

#include "common.hpp"
#include "replay_kernels.hpp"
#include "trainer.hpp"

namespace rp {
namespace {

constexpr unsigned int kThreads = kTrainThreads;

// ----------------------------------------------------------------------------- dense products
enum { EPI_NONE = 0, EPI_BIAS_RELU = 1, EPI_BIAS = 2, EPI_MASK = 3 };

// C[M x N] = op(A) op(B), 64 x 64 tile per block, fp32 accumulation in registers.
// op(A)(m,k) = TRANS_A ? A[k*lda + m] : A[m*lda + k];  op(B)(k,n) = TRANS_B ? B[n*ldb + k] : B[k*ldb + n].
template <typename TA, typename TB, typename TC, bool TRANS_A, bool TRANS_B, int EPI>
__global__ __launch_bounds__(kThreads) void gemm_kernel(int M, int N, int K,
                                                        const TA* __restrict__ A, int lda,
                                                        const TB* __restrict__ B, int ldb,
                                                        TC* __restrict__ C, int ldc,
                                                        const float* __restrict__ bias,
                                                        const TC* __restrict__ mask, int ldmask) {
    constexpr int BM = 64, BN = 64, BK = 16;
    __shared__ float As[BK][BM + 4];
    __shared__ float Bs[BK][BN + 4];
    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;
    const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
    float acc[4][4] = {};

    for (int k0 = 0; k0 < K; k0 += BK) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            int m, k;
            if (TRANS_A) { m = tid & 63; k = (tid >> 6) + 4 * j; }
            else         { k = tid & 15; m = (tid >> 4) + 16 * j; }
            const int gm = m0 + m, gk = k0 + k;
            float v = 0.f;
            if (gm < M && gk < K)
                v = to_float(TRANS_A ? A[(size_t)gk * lda + gm] : A[(size_t)gm * lda + gk]);
            As[k][m] = v;
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            int n, k;
            if (TRANS_B) { k = tid & 15; n = (tid >> 4) + 16 * j; }
            else         { n = tid & 63; k = (tid >> 6) + 4 * j; }
            const int gn = n0 + n, gk = k0 + k;
            float v = 0.f;
            if (gn < N && gk < K)
                v = to_float(TRANS_B ? B[(size_t)gn * ldb + gk] : B[(size_t)gk * ldb + gn]);
            Bs[k][n] = v;
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < BK; ++k) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = As[k][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) b[j] = Bs[k][tx * 4 + j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int gm = m0 + ty * 4 + i;
        if (gm >= M) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int gn = n0 + tx * 4 + j;
            if (gn >= N) continue;
            float v = acc[i][j];
            if (EPI == EPI_BIAS_RELU) {
                v += bias[gn];
                v = v > 0.f ? v : 0.f;
            } else if (EPI == EPI_BIAS) {
                v += bias[gn];
            } else if (EPI == EPI_MASK) {
                if (!(to_float(mask[(size_t)gm * ldmask + gn]) > 0.f)) v = 0.f;
            }
            C[(size_t)gm * ldc + gn] = from_float<TC>(v);
        }
    }
}

// out[n] = sum_m X[m*ld + n], rows added in order
template <typename T>
__global__ __launch_bounds__(kThreads) void colsum_kernel(int M, int N, const T* __restrict__ X,
                                                          int ld, float* __restrict__ out) {
    const int n = blockIdx.x * kThreads + threadIdx.x;
    if (n >= N) return;
    float acc = 0.f;
    for (int m = 0; m < M; ++m) acc += to_float(X[(size_t)m * ld + n]);
    out[n] = acc;
}

// ----------------------------------------------------------------------------- TD target and loss
// One wavefront per batch row i:  y_i = r_i + gamma (1 - term_i) max_a Q[B+i][a],
// delta_i = y_i - Q[i][a_i], per-sample loss, and the one non-zero of dL/dQ in row i.
// Thread 0 of block 0 also advances Adam's step count and its bias corrections.
__global__ __launch_bounds__(kThreads) void td_loss_kernel(
    unsigned int B, unsigned int A, unsigned int Ap, const float* __restrict__ Q,
    const int* __restrict__ act, const float* __restrict__ rew,
    const unsigned char* __restrict__ term, float gamma, unsigned int loss_kind,
    float* __restrict__ y_out, float* __restrict__ delta_out, float* __restrict__ lossi,
    float* __restrict__ dQ, TrainCounters* __restrict__ ctr, float beta1, float beta2) {
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        // (running products beta^t in double precision: no power function on the device)
        const double pw1 = ctr->pw1 * (double)beta1, pw2 = ctr->pw2 * (double)beta2;
        ctr->adam_t = ctr->adam_t + 1;
        ctr->pw1 = pw1;
        ctr->pw2 = pw2;
        ctr->c1 = (float)(1.0 - pw1);
        ctr->c2 = (float)(1.0 - pw2);
    }
    const unsigned int lane = threadIdx.x & 63u;
    const unsigned int i = blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
    if (i >= B) return;
    const float* qn = Q + (size_t)(B + i) * Ap;
    float best = -INFINITY;
    for (unsigned int k = lane; k < A; k += 64) best = fmaxf(best, qn[k]);
    best = wave_max(best);
    unsigned int ai = (unsigned int)act[i];
    if (ai >= A) ai = A - 1;  // an out-of-range action must not turn into a wild address
    const float q = Q[(size_t)i * Ap + ai];
    const float y = rew[i] + (term[i] ? 0.f : gamma * best);
    const float d = y - q;
    float li, slope;
    if (loss_kind == RP_MSE || fabsf(d) <= 1.f) {
        li = 0.5f * d * d;
        slope = d;
    } else {
        li = fabsf(d) - 0.5f;
        slope = d > 0.f ? 1.f : -1.f;
    }
    const float g = -slope / (float)B;
    for (unsigned int k = lane; k < Ap; k += 64) dQ[(size_t)i * Ap + k] = (k == ai) ? g : 0.f;
    if (lane == 0) {
        y_out[i] = y;
        delta_out[i] = d;
        lossi[i] = li;
    }
}

// dZ2[i][k] = dQ[i][a_i] * W3[k][a_i] * 1[H2[i][k] > 0]   (dQ has one non-zero per row)
template <typename E>
__global__ __launch_bounds__(kThreads) void dz_out_kernel(unsigned int B, unsigned int H,
                                                          unsigned int A, unsigned int Ap,
                                                          const float* __restrict__ dQ,
                                                          const int* __restrict__ act,
                                                          const E* __restrict__ W3,
                                                          const E* __restrict__ H2,
                                                          E* __restrict__ dZ2) {
    const size_t e = (size_t)blockIdx.x * kThreads + threadIdx.x;
    if (e >= (size_t)B * H) return;
    const unsigned int i = (unsigned int)(e / H), k = (unsigned int)(e - (size_t)i * H);
    unsigned int ai = (unsigned int)act[i];
    if (ai >= A) ai = A - 1;
    float v = dQ[(size_t)i * Ap + ai] * to_float(W3[(size_t)k * Ap + ai]);
    if (!(to_float(H2[e]) > 0.f)) v = 0.f;
    dZ2[e] = from_float<E>(v);
}

// ----------------------------------------------------------------------------- optimizer
// SGD or Adam over the flat parameter array; in mixed precision also refreshes the bf16 copy.
// Block 0 additionally reduces the per-sample losses to their mean and advances the
// sampling step counter.
__global__ __launch_bounds__(kThreads) void optimizer_kernel(
    unsigned int n, float* __restrict__ w, const float* __restrict__ g, float* __restrict__ m,
    float* __restrict__ v, bf16_t* __restrict__ wb, unsigned int opt, float lr, float beta1,
    float beta2, float eps, TrainCounters* __restrict__ ctr, const float* __restrict__ lossi,
    unsigned int B, float* __restrict__ wt, bf16_t* __restrict__ wbt, unsigned int sync_every) {
    const unsigned int k = blockIdx.x * kThreads + threadIdx.x;
    if (k < n) {
        float wk = w[k];
        const float gk = g[k];
        if (opt == RP_SGD) {
            wk -= lr * gk;
        } else {
            const float mk = beta1 * m[k] + (1.f - beta1) * gk;
            const float vk = beta2 * v[k] + (1.f - beta2) * gk * gk;
            m[k] = mk;
            v[k] = vk;
            wk -= lr * (mk / ctr->c1) / (sqrtf(vk / ctr->c2) + eps);
        }
        w[k] = wk;
        if (wb) wb[k] = from_float<bf16_t>(wk);
        // the frozen target network takes the new weights when the update count says so
        if (wt && sync_every && ctr->adam_t % sync_every == 0) {
            wt[k] = wk;
            if (wbt) wbt[k] = from_float<bf16_t>(wk);
        }
    }
    if (blockIdx.x == 0 && threadIdx.x < 64) {
        float acc = 0.f;
        for (unsigned int i = threadIdx.x; i < B; i += 64) acc += lossi[i];
        acc = wave_sum(acc);
        if (threadIdx.x == 0) {
            ctr->loss = acc / (float)B;
            ctr->step += 1;
        }
    }
}

// A caller-provided batch (structure of arrays, B rows) into the step's input buffers:
// X = [S ; S'] with row pitch Dp, the per-row fields, the batch position as "slot", and, for the
// MFMA step, the transposed copy of S.  E = element type of a state (4 or 2 bytes).
template <typename E>
__global__ __launch_bounds__(kThreads) void load_batch_kernel(
    unsigned int B, unsigned int D, unsigned int Dp, const E* __restrict__ s,
    const E* __restrict__ s_next, const int* __restrict__ a, const float* __restrict__ r,
    const unsigned char* __restrict__ term, E* __restrict__ X, E* __restrict__ XT,
    unsigned int ldt, int* __restrict__ act, float* __restrict__ rew,
    unsigned char* __restrict__ trm, unsigned int* __restrict__ idx) {
    const size_t e = (size_t)blockIdx.x * kThreads + threadIdx.x;
    if (e < (size_t)B * D) {
        const unsigned int i = (unsigned int)(e / D), c = (unsigned int)(e - (size_t)i * D);
        const E v = s[e];
        X[(size_t)i * Dp + c] = v;
        X[(size_t)(B + i) * Dp + c] = s_next[e];
        if (XT) XT[(size_t)c * ldt + i] = v;
    }
    if (e < B) {
        act[e] = a[e];
        rew[e] = r[e];
        trm[e] = term[e] ? 1 : 0;
        idx[e] = (unsigned int)e;
    }
}

__global__ __launch_bounds__(kThreads) void to_bf16_kernel(unsigned int n,
                                                           const float* __restrict__ w,
                                                           bf16_t* __restrict__ wb) {
    const unsigned int k = blockIdx.x * kThreads + threadIdx.x;
    if (k < n) wb[k] = from_float<bf16_t>(w[k]);
}

}  // namespace
}  // namespace rp

using rp::bf16_t;
using rp::TrainCounters;

namespace rp {
namespace {

struct WsLayout {
    size_t ctr, w, g, m, v, wt, w2t, wb, wbt, X, act, rew, term, idx, H1, H2, Q, y, delta, lossi, dQ, dZ2, dZ1,
        pre, qpart, handoff, ahead, qn_ahead, X2, total;
    // mixed-precision step on MFMA
    size_t W1T, W2b, W2T, W3T, W1Tt, W2Tt, W3Tt, XT, H1T, H2T, dQTh, dQTl, dZ2T, dZ1T, part3, part1, part2;
    unsigned int Dp, Ap, Bp;
    size_t n_params, n_padded, n_head, elem;
    size_t oW1, ob1, oW2, ob2, oW3, ob3;
};

bool ws_layout(const train_config* c, WsLayout* L) {
    if (!c || c->state_dim == 0 || c->state_dim > 4096 || c->hidden == 0 || c->hidden % 64 != 0 ||
        c->hidden > 8192 || c->hidden2 % 64 != 0 || c->hidden2 > 8192 || c->num_actions == 0 ||
        c->num_actions > 4096 || c->batch == 0 ||
        c->batch > (1u << 20) || (c->param_dtype != RP_F32 && c->param_dtype != RP_BF16) ||
        c->loss > RP_MSE || c->opt > RP_ADAM || c->head > RP_HEAD_DUELING)
        return false;
    // H, G: widths of the first and the second hidden layer
    const size_t D = c->state_dim, H = c->hidden, G = c->hidden2 ? c->hidden2 : c->hidden;
    const size_t A = c->num_actions, B = c->batch;
    L->Dp = (unsigned int)align_up(D, 32);
    L->Ap = (unsigned int)align_up(A, 32);
    L->elem = c->param_dtype == RP_BF16 ? 2 : 4;
    const size_t O = c->head == RP_HEAD_DUELING ? A + 1 : A;   // outputs of the last layer
    L->n_params = D * H + H + H * G + G + G * O + O;
    L->n_head = c->head == RP_HEAD_DUELING ? (G + 1) * O : 0;
    L->oW1 = 0;
    L->ob1 = L->oW1 + (size_t)L->Dp * H;
    L->oW2 = L->ob1 + H;
    L->ob2 = L->oW2 + H * G;
    L->oW3 = L->ob2 + G;
    L->ob3 = L->oW3 + G * L->Ap;
    L->n_padded = L->ob3 + L->Ap;
    size_t o = 0;
    auto take = [&](size_t bytes) {
        size_t at = o;
        o = align_up(o + bytes, 256);
        return at;
    };
    L->ctr = take(sizeof(TrainCounters));
    const size_t n_dev = L->n_padded + L->n_head;
    L->w = take(n_dev * 4);
    L->g = take(n_dev * 4);
    L->m = take(n_dev * 4);
    L->v = take(n_dev * 4);
    L->wt = take(c->target_sync ? n_dev * 4 : 0);
    L->w2t = take(c->param_dtype == RP_F32 ? G * H * 4 : 0);
    L->wb = take(c->param_dtype == RP_BF16 ? L->n_padded * 2 : 0);
    L->wbt = take(c->param_dtype == RP_BF16 && c->target_sync ? L->n_padded * 2 : 0);
    L->X = take(2 * B * L->Dp * L->elem);
    // (a second batch buffer for the fp32 step on MFMA, whose weights kernel still reads the batch
    // while its extra workgroups gather the next one)
    L->X2 = take(c->param_dtype == RP_F32 ? 2 * B * L->Dp * L->elem : 0);
    L->act = take(B * 4);
    L->rew = take(B * 4);
    L->term = take(B);
    L->idx = take(B * 4);
    L->H1 = take(2 * B * H * L->elem);
    L->H2 = take(2 * B * G * L->elem);
    L->Q = take(2 * B * L->Ap * 4);
    L->y = take(B * 4);
    L->delta = take(B * 4);
    L->lossi = take(B * 4);
    L->dQ = take(B * L->Ap * 4);
    L->dZ2 = take(B * G * L->elem);
    L->dZ1 = take(B * H * L->elem);
    L->pre = take(2 * (4 + B) * 4);
    // (partial products of the output layer, fp32 step on MFMA: up to 8 per element)
    L->qpart = take(c->param_dtype == RP_F32 ? 8 * 2 * B * L->Ap * 4 : 0);
    L->handoff = take(c->target_sync ? B * 8 : 0);
    L->ahead = take(c->target_sync ? 2 * B * 8 * 4 : 0);
    L->qn_ahead = take(c->target_sync ? 2 * B * L->Ap * 4 : 0);
    // the MFMA mixed-precision step exists for two hidden layers of one width
    const bool mixed = c->param_dtype == RP_BF16 && H == G;
    const size_t Bp = align_up(B, 128), Dx = align_up(D + 1, 32);
    L->Bp = (unsigned int)Bp;
    L->W1T = take(mixed ? H * L->Dp * 2 : 0);
    L->W2b = take(mixed ? H * H * 2 : 0);
    L->W2T = take(mixed ? H * H * 2 : 0);
    L->W3T = take(mixed ? L->Ap * H * 2 : 0);
    const bool mixed_t = mixed && c->target_sync;
    L->W1Tt = take(mixed_t ? H * L->Dp * 2 : 0);
    L->W2Tt = take(mixed_t ? H * H * 2 : 0);
    L->W3Tt = take(mixed_t ? L->Ap * H * 2 : 0);
    L->XT = take(mixed ? Dx * Bp * 2 : 0);
    L->H1T = take(mixed ? (H + 1) * Bp * 2 : 0);
    L->H2T = take(mixed ? (H + 1) * Bp * 2 : 0);
    L->dQTh = take(mixed ? 2 * L->Ap * Bp * 2 : 0);   // high part, then low part
    L->dQTl = L->dQTh + L->Ap * Bp * 2;
    L->dZ2T = take(mixed ? H * Bp * 2 : 0);
    L->dZ1T = take(mixed ? H * Bp * 2 : 0);
    // K-split partial products of the narrow layers' gradients (at most 16 splits)
    L->part3 = take(mixed ? 16 * (H + 1) * 2 * L->Ap * 4 : 0);
    L->part1 = take(mixed ? 16 * H * Dx * 4 : 0);
    L->part2 = take(mixed ? (size_t)square_splits((unsigned int)Bp, (unsigned int)H) * (H + 1) * H * 4 : 0);
    L->total = o;
    return true;
}

// external [W1 b1 W2 b2 W3 b3] <-> device order: padded arrays (zero rows / columns as padding)
// and, for the dueling head, its own parameters behind them.  `weights`: also fill positions
// W3 / b3 of the padded part with the plain output layer the dueling head amounts to.
void pad_params(const trainer* t, const float* ext, std::vector<float>& pad, bool weights = true) {
    const size_t D = t->cfg.state_dim, H = t->H, G = t->Hb, A = t->cfg.num_actions, Ap = t->Ap;
    pad.assign(t->n_dev, 0.f);
    const float* p = ext;
    memcpy(&pad[t->oW1], p, D * H * 4); p += D * H;
    memcpy(&pad[t->ob1], p, H * 4);     p += H;
    memcpy(&pad[t->oW2], p, H * G * 4); p += H * G;
    memcpy(&pad[t->ob2], p, G * 4);     p += G;
    if (!t->dueling) {
        for (size_t k = 0; k < G; ++k) memcpy(&pad[t->oW3 + k * Ap], p + k * A, A * 4);
        p += G * A;
        memcpy(&pad[t->ob3], p, A * 4);
        return;
    }
    const size_t O = A + 1;
    float* head = &pad[t->n_padded];
    memcpy(head, p, (G + 1) * O * 4);          // W3[G x O] followed by b3[O] = [(G+1) x O]
    if (!weights) return;
    for (size_t k = 0; k <= G; ++k) {
        const float* row = head + k * O;
        const float v = head_connected((unsigned int)G, (unsigned int)k, 0) ? row[0] : 0.f;
        const bool adv_on = head_connected((unsigned int)G, (unsigned int)k, 1);
        float sum = 0.f;
        for (size_t a = 0; a < A; ++a) sum += adv_on ? row[1 + a] : 0.f;
        const float mean = sum / (float)A;
        float* dst = k < G ? &pad[t->oW3 + k * Ap] : &pad[t->ob3];
        for (size_t a = 0; a < A; ++a) dst[a] = v + (adv_on ? row[1 + a] : 0.f) - mean;
    }
}

void unpad_params(const trainer* t, const std::vector<float>& pad, float* ext) {
    const size_t D = t->cfg.state_dim, H = t->H, G = t->Hb, A = t->cfg.num_actions, Ap = t->Ap;
    float* p = ext;
    memcpy(p, &pad[t->oW1], D * H * 4); p += D * H;
    memcpy(p, &pad[t->ob1], H * 4);     p += H;
    memcpy(p, &pad[t->oW2], H * G * 4); p += H * G;
    memcpy(p, &pad[t->ob2], G * 4);     p += G;
    if (t->dueling) {
        memcpy(p, &pad[t->n_padded], (G + 1) * (A + 1) * 4);
        return;
    }
    for (size_t k = 0; k < G; ++k) memcpy(p + k * A, &pad[t->oW3 + k * Ap], A * 4);
    p += G * A;
    memcpy(p, &pad[t->ob3], A * 4);
}

// ----------------------------------------------------------------------------- dueling head
// One wavefront per hidden unit k (k = H: the biases).  g holds the gradient of the equivalent
// plain output layer, dW[k][a]; the head's own gradients follow from the combine
// Q = V + A - mean A:  dV[k] = sum_a dW[k][a],  dA[k][a] = dW[k][a] - mean_a' dW[k][a'],
// restricted to the weights the head has.  After the optimizer step the equivalent layer is
// rebuilt, with its bf16 copies, and the target network takes it all when a sync is due.
struct HeadArgs {
    unsigned int H, A, Ap;
    size_t oW3, ob3, n_padded;
    float *w, *g, *m, *v, *wt;
    unsigned int opt, sync_every;
    float lr, beta1, beta2, eps;
    const TrainCounters* ctr;
    unsigned short *W3T, *W3T_t;   // MFMA step: [Ap x H] operand copies (trained / target)
    bf16_t *wb, *wbt;              // layered mixed precision: padded bf16 copies
};

__global__ __launch_bounds__(64) void dueling_head_kernel(HeadArgs p) {
    // one single-wavefront workgroup per hidden unit k, one lane per output (striding when there
    // are more than 64); the new head weights of the row pass through LDS
    extern __shared__ float head_row[];   // [1 + A]
    const unsigned int lane = threadIdx.x;
    const unsigned int k = blockIdx.x;
    const unsigned int A = p.A, O = A + 1;
    const size_t eff = k < p.H ? p.oW3 + (size_t)k * p.Ap : p.ob3;   // row k of the plain layer
    const size_t head = p.n_padded + (size_t)k * O;
    const bool v_on = head_connected(p.H, k, 0), a_on = head_connected(p.H, k, 1);
    const float c1 = p.ctr->c1, c2 = p.ctr->c2;
    const bool sync = p.wt && p.sync_every && p.ctr->adam_t % p.sync_every == 0;

    float part = 0.f;
    for (unsigned int a = lane; a < A; a += 64) part += p.g[eff + a];
    const float gsum = wave_sum(part);
    const float gmean = gsum / (float)A;
    float vpart = 0.f, apart = 0.f;
    for (unsigned int o = lane; o < O; o += 64) {
        const bool on = o == 0 ? v_on : a_on;
        const float gk = !on ? 0.f : o == 0 ? gsum : p.g[eff + o - 1] - gmean;
        float wk = p.w[head + o];
        p.g[head + o] = gk;
        if (on) {
            if (p.opt == RP_SGD) {
                wk -= p.lr * gk;
            } else {
                const float mk = p.beta1 * p.m[head + o] + (1.f - p.beta1) * gk;
                const float vk = p.beta2 * p.v[head + o] + (1.f - p.beta2) * gk * gk;
                p.m[head + o] = mk;
                p.v[head + o] = vk;
                wk -= p.lr * (mk / c1) / (sqrtf(vk / c2) + p.eps);
            }
            p.w[head + o] = wk;
            if (o == 0) vpart = wk; else apart += wk;
        }
        head_row[o] = on ? wk : 0.f;
        if (sync) p.wt[head + o] = wk;
    }
    // the new value weight sits in lane 0, the advantage weights are spread over the lanes
    const float vnew = wave_sum(vpart);
    const float amean = wave_sum(apart) / (float)A;
    // (LDS operations of a wavefront complete in order: the row is there)
    for (unsigned int a = lane; a < A; a += 64) {
        const float e = vnew + head_row[1 + a] - amean;
        p.w[eff + a] = e;
        if (p.wb) p.wb[eff + a] = from_float<bf16_t>(e);
        if (p.W3T && k < p.H) p.W3T[(size_t)a * p.H + k] = bf16_bits_rne(e);
        if (sync) {
            p.wt[eff + a] = e;
            if (p.wbt) p.wbt[eff + a] = from_float<bf16_t>(e);
            if (p.W3T_t && k < p.H) p.W3T_t[(size_t)a * p.H + k] = bf16_bits_rne(e);
        }
    }
}

template <typename TA, typename TB, typename TC, bool TRA, bool TRB, int EPI>
void gemm(hipStream_t st, int M, int N, int K, const void* A, int lda, const void* B, int ldb,
          void* C, int ldc, const float* bias, const void* mask, int ldmask) {
    dim3 grid((N + 63) / 64, (M + 63) / 64);
    hipLaunchKernelGGL((gemm_kernel<TA, TB, TC, TRA, TRB, EPI>), grid, dim3(kThreads), 0, st, M, N,
                       K, static_cast<const TA*>(A), lda, static_cast<const TB*>(B), ldb,
                       static_cast<TC*>(C), ldc, bias, static_cast<const TC*>(mask), ldmask);
}

// Enqueue every kernel of one executed train step (after the append).  E is the element
// type of activations and of the matrices the products read.
template <typename E>
hipError_t enqueue_step(trainer* t, hipStream_t st, unsigned int* count, bool sample) {
    // H, G: widths of the first and the second hidden layer
    const int B = (int)t->B, H = (int)t->H, G = (int)t->Hb, Dp = (int)t->Dp, Ap = (int)t->Ap;
    const unsigned int A = t->cfg.num_actions;
    const bool mixed = t->cfg.param_dtype == RP_BF16;
    const unsigned char* wsrc = mixed ? reinterpret_cast<const unsigned char*>(t->wb)
                                      : reinterpret_cast<const unsigned char*>(t->w);
    const size_t eb = t->elem;
    const void* W1 = wsrc + t->oW1 * eb;
    const void* W2 = wsrc + t->oW2 * eb;
    const void* W3 = wsrc + t->oW3 * eb;
    unsigned int n = 0;

    // sample B slots with the device-resident step counter and unpack into X = [S ; S']
    hipError_t e = hipSuccess;
    unsigned int launched = 0;
    if (sample) {
        e = launch_sample_gather(t->rp_->geom, t->rp_->cfg.seed, 0, &t->ctr->step, t->B, t->X,
                                 static_cast<unsigned char*>(t->X) + (size_t)B * Dp * eb, t->Dp,
                                 t->act, t->rew, t->term, t->idx, st, nullptr, 0, 0, 0,
                                 t->rp_->draw_scratch, &launched);
        if (e != hipSuccess) return e;
        n += launched;
    }
    // forward on the 2B rows of X; with a frozen target network the rows of S' (B .. 2B-1) go
    // through its weights in launches of their own
    if (!t->wt) {
        gemm<E, E, E, false, false, EPI_BIAS_RELU>(st, 2 * B, H, Dp, t->X, Dp, W1, H, t->H1, H,
                                                   t->w + t->ob1, nullptr, 0); ++n;
        gemm<E, E, E, false, false, EPI_BIAS_RELU>(st, 2 * B, G, H, t->H1, H, W2, G, t->H2, G,
                                                   t->w + t->ob2, nullptr, 0); ++n;
        gemm<E, E, float, false, false, EPI_BIAS>(st, 2 * B, Ap, G, t->H2, G, W3, Ap, t->Q, Ap,
                                                  t->w + t->ob3, nullptr, 0); ++n;
    } else {
        const unsigned char* tsrc = mixed ? reinterpret_cast<const unsigned char*>(t->wbt)
                                          : reinterpret_cast<const unsigned char*>(t->wt);
        const unsigned char* Xb = static_cast<const unsigned char*>(t->X);
        unsigned char* H1b = static_cast<unsigned char*>(t->H1);
        unsigned char* H2b = static_cast<unsigned char*>(t->H2);
        for (int half = 0; half < 2; ++half) {
            const unsigned char* ws_ = half ? tsrc : wsrc;
            const float* bias = half ? t->wt : t->w;
            const size_t r0 = half ? (size_t)B : 0;
            gemm<E, E, E, false, false, EPI_BIAS_RELU>(st, B, H, Dp, Xb + r0 * Dp * eb, Dp,
                                                       ws_ + t->oW1 * eb, H, H1b + r0 * H * eb, H,
                                                       bias + t->ob1, nullptr, 0); ++n;
            gemm<E, E, E, false, false, EPI_BIAS_RELU>(st, B, G, H, H1b + r0 * H * eb, H,
                                                       ws_ + t->oW2 * eb, G, H2b + r0 * G * eb, G,
                                                       bias + t->ob2, nullptr, 0); ++n;
            gemm<E, E, float, false, false, EPI_BIAS>(st, B, Ap, G, H2b + r0 * G * eb, G,
                                                      ws_ + t->oW3 * eb, Ap, t->Q + r0 * Ap, Ap,
                                                      bias + t->ob3, nullptr, 0); ++n;
        }
    }
    // targets, TD errors, loss terms, dL/dQ
    hipLaunchKernelGGL(td_loss_kernel, dim3((B + 3) / 4), dim3(kThreads), 0, st, t->B, A, t->Ap,
                       t->Q, t->act, t->rew, t->term, t->cfg.gamma, t->cfg.loss, t->y, t->delta,
                       t->lossi, t->dQ, t->ctr, t->cfg.beta1, t->cfg.beta2); ++n;
    // output layer
    gemm<E, float, float, true, false, EPI_NONE>(st, G, Ap, B, t->H2, G, t->dQ, Ap,
                                                 t->g + t->oW3, Ap, nullptr, nullptr, 0); ++n;
    hipLaunchKernelGGL(colsum_kernel<float>, dim3((Ap + kThreads - 1) / kThreads), dim3(kThreads),
                       0, st, B, Ap, t->dQ, Ap, t->g + t->ob3); ++n;
    hipLaunchKernelGGL(dz_out_kernel<E>, dim3(((size_t)B * G + kThreads - 1) / kThreads),
                       dim3(kThreads), 0, st, t->B, t->Hb, A, t->Ap, t->dQ, t->act,
                       static_cast<const E*>(W3), static_cast<const E*>(t->H2),
                       static_cast<E*>(t->dZ2)); ++n;
    // second hidden layer
    gemm<E, E, float, true, false, EPI_NONE>(st, H, G, B, t->H1, H, t->dZ2, G, t->g + t->oW2, G,
                                             nullptr, nullptr, 0); ++n;
    hipLaunchKernelGGL(colsum_kernel<E>, dim3((G + kThreads - 1) / kThreads), dim3(kThreads), 0, st,
                       B, G, static_cast<const E*>(t->dZ2), G, t->g + t->ob2); ++n;
    gemm<E, E, E, false, true, EPI_MASK>(st, B, H, G, t->dZ2, G, W2, G, t->dZ1, H, nullptr, t->H1,
                                         H); ++n;
    // first hidden layer
    gemm<E, E, float, true, false, EPI_NONE>(st, Dp, H, B, t->X, Dp, t->dZ1, H, t->g + t->oW1, H,
                                             nullptr, nullptr, 0); ++n;
    hipLaunchKernelGGL(colsum_kernel<E>, dim3((H + kThreads - 1) / kThreads), dim3(kThreads), 0, st,
                       B, H, static_cast<const E*>(t->dZ1), H, t->g + t->ob1); ++n;
    // update
    // (with the dueling head the output layer's update belongs to the head kernel)
    const unsigned int n_opt = (unsigned int)(t->dueling ? t->oW3 : t->n_padded);
    hipLaunchKernelGGL(optimizer_kernel, dim3((n_opt + kThreads - 1) / kThreads),
                       dim3(kThreads), 0, st, n_opt, t->w, t->g, t->m, t->v,
                       t->wb, t->cfg.opt, t->cfg.lr, t->cfg.beta1, t->cfg.beta2, t->cfg.eps, t->ctr,
                       t->lossi, t->B, t->wt, t->wbt, t->cfg.target_sync); ++n;
    unsigned int nh = 0;
    e = enqueue_head_update(t, st, &nh);
    if (e != hipSuccess) return e;
    if (count) *count = n + nh;
    return hipGetLastError();
}

// Enqueue one executed step: the kernel that consumes the new experiences first.
hipError_t enqueue_append_and_step(trainer* t, const Payload& src, hipStream_t st,
                                   unsigned int* count) {
    if (t->fused) return enqueue_fused_step(t, src, nullptr, st, count);
    unsigned int n = 0, k = 0;
    replay* r = t->rp_;
    if (t->cfg.appends_per_step && (t->wide || t->mid)) {
        // append, sample and gather in one launch; the step then starts from the gathered batch
        const unsigned int Dp = t->Dp;
        unsigned char* X = static_cast<unsigned char*>(t->X);
        t->append_args = make_append_gather_args(
            r->geom, RingPos{r->head, r->size, r->total}, t->cfg.appends_per_step, src, r->cfg.seed,
            nullptr, t->B,
            GatherOut{X, X + (size_t)t->B * Dp * t->elem, Dp, t->act, t->rew, t->term, t->idx,
                      t->wide ? t->wd.XT : nullptr, t->Bp});
        t->append_args.step_value = t->host_step;   // (the host mirrors the device's counter exactly)
        unsigned int blocks;
        size_t lds;
        append_gather_shape(t->append_args, &blocks, &lds);
        void* kargs[] = {&t->append_args};
        // (in a recorded run the step before this one may have gathered this step's batch already)
        hipError_t e = t->rec_skip_gather ? hipSuccess
                                          : hipLaunchKernel(append_gather_func(r->geom), dim3(blocks),
                                                            dim3(kThreads), kargs, lds, st);
        if (e != hipSuccess) return e;
        e = t->wide ? enqueue_wide_step(t, st, &k, false) : enqueue_mid_step(t, st, &k);
        if (count) *count = 1 + k;
        return e;
    }
    if (t->cfg.appends_per_step) {
        static_cast<AppendArgs&>(t->append_args) =
            make_append_args(r->geom, RingPos{r->head, r->size, r->total}, t->cfg.appends_per_step, src);
        void* kargs[] = {&t->append_args};
        hipError_t e = hipLaunchKernel(append_pair_func(r->geom), dim3(append_blocks(t->append_args)),
                                       dim3(kThreads), kargs, 0, st);
        if (e != hipSuccess) return e;
        ++n;
    }
    if (t->mid) {
        // (no new experiences per step: sample and gather on their own, then the step)
        unsigned int launched = 0;
        hipError_t e = launch_sample_gather(r->geom, r->cfg.seed, 0, &t->ctr->step, t->B, t->X,
                                            static_cast<unsigned char*>(t->X) + (size_t)t->B * t->Dp * 4, t->Dp,
                                            t->act, t->rew, t->term, t->idx, st, nullptr, 0, 0, 0,
                                            r->draw_scratch, &launched);
        if (e != hipSuccess) return e;
        e = enqueue_mid_step(t, st, &k);
        if (count) *count = n + launched + k;
        return e;
    }
    hipError_t e = t->wide ? enqueue_wide_step(t, st, &k, true)
                   : t->cfg.param_dtype == RP_BF16 ? enqueue_step<bf16_t>(t, st, &k, true)
                                                   : enqueue_step<float>(t, st, &k, true);
    if (count) *count = n + k;
    return e;
}

// Enqueue one step on a caller-provided batch (device arrays): no append, no sampling.
hipError_t enqueue_batch_step(trainer* t, const Payload& batch, hipStream_t st) {
    if (t->fused) return enqueue_fused_step(t, Payload{nullptr, nullptr, nullptr, nullptr, nullptr},
                                            &batch, st, nullptr);
    const unsigned int B = t->B, D = t->cfg.state_dim;
    const unsigned int blocks = (unsigned int)(((size_t)B * D + kThreads - 1) / kThreads);
    if (t->cfg.param_dtype == RP_BF16) {
        typedef unsigned short E;
        hipLaunchKernelGGL(load_batch_kernel<E>, dim3(blocks), dim3(kThreads), 0, st, B, D, t->Dp,
                           reinterpret_cast<const E*>(batch.s), reinterpret_cast<const E*>(batch.s_next),
                           batch.a, batch.r, batch.term, static_cast<E*>(t->X),
                           t->wide ? t->wd.XT : nullptr, t->Bp, t->act, t->rew, t->term, t->idx);
    } else {
        hipLaunchKernelGGL(load_batch_kernel<float>, dim3(blocks), dim3(kThreads), 0, st, B, D, t->Dp,
                           reinterpret_cast<const float*>(batch.s),
                           reinterpret_cast<const float*>(batch.s_next), batch.a, batch.r, batch.term,
                           static_cast<float*>(t->X), static_cast<float*>(nullptr), 0u, t->act,
                           t->rew, t->term, t->idx);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    return t->wide  ? enqueue_wide_step(t, st, nullptr, false)
           : t->mid ? enqueue_mid_step(t, st, nullptr)
           : t->cfg.param_dtype == RP_BF16 ? enqueue_step<bf16_t>(t, st, nullptr, false)
                                           : enqueue_step<float>(t, st, nullptr, false);
}

// Find the nodes of the payload-consuming kernel in a recorded graph, in execution order (the
// graph is a chain: one root, every node one dependent).  Finds `want` of them or fails.
hipError_t find_kernel_nodes(trainer* t, hipGraph_t graph, const void* func, unsigned int want,
                             hipGraphNode_t* nodes, hipKernelNodeParams* params) {
    size_t n_roots = 0;
    hipError_t e = hipGraphGetRootNodes(graph, nullptr, &n_roots);
    if (e != hipSuccess) return e;
    if (n_roots != 1) return hipErrorInvalidValue;
    hipGraphNode_t cur = nullptr;
    e = hipGraphGetRootNodes(graph, &cur, &n_roots);
    if (e != hipSuccess) return e;
    unsigned int found = 0;
    for (;;) {
        hipGraphNodeType type;
        e = hipGraphNodeGetType(cur, &type);
        if (e != hipSuccess) return e;
        if (type == hipGraphNodeTypeKernel) {
            hipKernelNodeParams np;
            e = hipGraphKernelNodeGetParams(cur, &np);
            if (e != hipSuccess) return e;
            if (np.func == func && found < want) {
                nodes[found] = cur;
                params[found] = np;
                params[found].kernelParams = t->payload_kargs;
                params[found].extra = nullptr;
                ++found;
            }
        }
        size_t n_next = 0;
        e = hipGraphNodeGetDependentNodes(cur, nullptr, &n_next);
        if (e != hipSuccess) return e;
        if (n_next == 0) break;
        if (n_next != 1) return hipErrorInvalidValue;
        hipGraphNode_t next = nullptr;
        e = hipGraphNodeGetDependentNodes(cur, &next, &n_next);
        if (e != hipSuccess) return e;
        cur = next;
    }
    return found == want ? hipSuccess : hipErrorNotFound;
}

hipError_t find_payload_nodes(trainer* t, hipGraph_t graph, unsigned int want, hipGraphNode_t* nodes,
                              hipKernelNodeParams* params) {
    return find_kernel_nodes(t, graph, t->payload_func, want, nodes, params);
}

// Whether a recorded step has a node whose argument changes from step to step.
bool has_payload_node(const trainer* t) { return t->fused || t->cfg.appends_per_step != 0; }

// Point the payload kernel's argument block at step `k` steps ahead of the host mirrors.
void set_payload_args(trainer* t, const Payload& src, unsigned int k) {
    const replay* r = t->rp_;
    const uint64_t n = t->cfg.appends_per_step, cap = r->cfg.capacity;
    const uint64_t head = (r->head + k * n) % cap;
    const uint64_t size = r->size + k * n > cap ? cap : r->size + k * n;
    const uint64_t total = r->total + k * n;
    if (t->fused) {
        t->row_args.src = src;
        t->row_args.n_append = (unsigned int)n;
        t->row_args.from_batch = 0;
        t->row_args.head = head;
        t->row_args.step = t->host_step + k;
        t->row_args.size_after = (unsigned int)(size + n > cap ? cap : size + n);
        t->row_args.next_size = (unsigned int)(size + 2 * n > cap ? cap : size + 2 * n);
        t->row_args.total_after = total + n;
        rp::set_adam_step(t->row_args, t->host_adam_t + k + 1, t->cfg.beta1, t->cfg.beta2);
        rp::stamp_launch(t, t->row_args);
    } else {
        t->append_args.src = src;
        t->append_args.pos = RingPos{head, size, total};
        t->append_args.step_value = t->host_step + k;
        if (t->gather_ahead) {
            // (the steps of a recorded run alternate between the two batch buffers)
            unsigned char* X = static_cast<unsigned char*>(t->X_buf[k & 1u]);
            t->append_args.out.out_s = X;
            t->append_args.out.out_s_next = X + (size_t)t->B * t->Dp * t->elem;
        }
    }
}

}  // namespace

hipError_t enqueue_head_update(trainer* t, hipStream_t st, unsigned int* count) {
    if (count) *count = 0;
    if (!t->dueling) return hipSuccess;
    HeadArgs a;
    a.H = t->Hb; a.A = t->cfg.num_actions; a.Ap = t->Ap;
    a.oW3 = t->oW3; a.ob3 = t->ob3; a.n_padded = t->n_padded;
    a.w = t->w; a.g = t->g; a.m = t->m; a.v = t->v; a.wt = t->wt;
    a.opt = t->cfg.opt; a.sync_every = t->cfg.target_sync;
    a.lr = t->cfg.lr; a.beta1 = t->cfg.beta1; a.beta2 = t->cfg.beta2; a.eps = t->cfg.eps;
    a.ctr = t->ctr;
    a.W3T = t->wide ? t->wd.W3T : nullptr;
    a.W3T_t = t->wide && t->wt ? t->wd.W3T_t : nullptr;
    a.wb = t->wide ? nullptr : t->wb;
    a.wbt = t->wide ? nullptr : t->wbt;
    hipLaunchKernelGGL(dueling_head_kernel, dim3(t->Hb + 1), dim3(64),
                       (t->cfg.num_actions + 1) * sizeof(float), st, a);
    if (count) *count = 1;
    return hipGetLastError();
}

// Host-sourced payloads: the experiences of one step are copied into the next pinned,
// device-mapped slot, which the payload kernel then reads in place over the host link.  Slots
// are reused in a ring; one event per group of kPinGroup slots tells when the kernels that read
// the group have finished.  stage_host_payload fills slot pin_next + ahead and returns the
// device view of it; commit_host_slots is called after the launch(es) that read `count` slots.
hipError_t stage_host_payload(trainer* t, unsigned int ahead, uint64_t n, const void* s,
                              const void* s_next, const int32_t* a, const float* r,
                              const uint8_t* term, Payload* out) {
    const unsigned int slot = (unsigned int)((t->pin_next + ahead) % kPinSlots);
    const unsigned int grp = slot / kPinGroup;
    if (slot % kPinGroup == 0 && t->pin_event_live[grp]) {
        hipError_t e = hipEventSynchronize(t->pin_event[grp]);
        if (e != hipSuccess) return e;
    }
    const size_t sb = t->rp_->geom.state_bytes, base = (size_t)slot * t->pin_slot_bytes;
    unsigned char* h = t->pin_host + base;
    memcpy(h, s, n * sb);
    memcpy(h + t->pin_off_s_next, s_next, n * sb);
    memcpy(h + t->pin_off_a, a, n * 4);
    memcpy(h + t->pin_off_r, r, n * 4);
    memcpy(h + t->pin_off_term, term, n);
    const unsigned char* d = t->pin_dev + base;
    *out = Payload{d, d + t->pin_off_s_next, reinterpret_cast<const int*>(d + t->pin_off_a),
                   reinterpret_cast<const float*>(d + t->pin_off_r), d + t->pin_off_term};
    return hipSuccess;
}

hipError_t commit_host_slots(trainer* t, unsigned int count, hipStream_t st) {
    for (unsigned int c = 0; c < count; ++c) {
        const unsigned int slot = (unsigned int)(t->pin_next % kPinSlots);
        if (slot % kPinGroup == kPinGroup - 1) {
            const unsigned int grp = slot / kPinGroup;
            hipError_t e = hipEventRecord(t->pin_event[grp], st);
            if (e != hipSuccess) return e;
            t->pin_event_live[grp] = true;
        }
        t->pin_next += 1;
    }
    return hipSuccess;
}

}  // namespace rp

extern "C" {

size_t train_param_count(const train_config* cfg) {
    rp::WsLayout L;
    return rp::ws_layout(cfg, &L) ? L.n_params : 0;
}

size_t train_workspace_bytes(const train_config* cfg) {
    rp::WsLayout L;
    return rp::ws_layout(cfg, &L) ? L.total : 0;
}

rp_status train_create(const train_config* cfg, replay_t* rp_, void* dev_workspace, size_t bytes,
                       const float* host_init_params, trainer_t** out) {
    RP_REQUIRE(cfg && rp_ && dev_workspace && host_init_params && out, "train_create: null argument");
    rp::WsLayout L;
    RP_REQUIRE(rp::ws_layout(cfg, &L),
               "train_create: invalid configuration (hidden and hidden2 must be multiples of 64; "
               "batch, state_dim, num_actions >= 1)");
    RP_REQUIRE(rp_->cfg.layout == RP_PAIR, "train_create: the trainer needs a PAIR replay");
    RP_REQUIRE(rp_->cfg.state_dim == cfg->state_dim, "train_create: state_dim %u != replay's %u",
               cfg->state_dim, rp_->cfg.state_dim);
    RP_REQUIRE((cfg->param_dtype == RP_F32 && rp_->cfg.state_dtype == RP_F32) ||
                   (cfg->param_dtype == RP_BF16 && rp_->cfg.state_dtype == RP_BF16),
               "train_create: param_dtype and the replay's state_dtype must both be F32 or both BF16");
    RP_REQUIRE(cfg->appends_per_step <= rp_->cfg.max_append && cfg->appends_per_step <= rp_->cfg.capacity,
               "train_create: appends_per_step %u exceeds the replay's max_append %u or capacity",
               cfg->appends_per_step, rp_->cfg.max_append);
    RP_REQUIRE((reinterpret_cast<uintptr_t>(dev_workspace) & 255u) == 0,
               "train_create: dev_workspace must be 256-byte aligned");
    if (bytes < L.total) {
        rp::set_error("train_create: workspace of %zu bytes is smaller than the %zu needed", bytes,
                      L.total);
        return RP_ENOMEM;
    }
    trainer* t = new (std::nothrow) trainer();
    if (!t) {
        rp::set_error("train_create: out of host memory");
        return RP_ENOMEM;
    }
    t->cfg = *cfg;
    t->rp_ = rp_;
    t->Dp = L.Dp; t->Ap = L.Ap; t->H = cfg->hidden; t->B = cfg->batch; t->Bp = L.Bp;
    t->Hb = cfg->hidden2 ? cfg->hidden2 : cfg->hidden;
    t->n_params = L.n_params; t->n_padded = L.n_padded; t->elem = L.elem;
    t->dueling = cfg->head == RP_HEAD_DUELING;
    t->n_head = L.n_head;
    t->n_dev = L.n_padded + L.n_head;
    t->oW1 = L.oW1; t->ob1 = L.ob1; t->oW2 = L.oW2; t->ob2 = L.ob2; t->oW3 = L.oW3; t->ob3 = L.ob3;
    unsigned char* ws = static_cast<unsigned char*>(dev_workspace);
    t->ws = ws;
    t->ctr = reinterpret_cast<TrainCounters*>(ws + L.ctr);
    t->w = reinterpret_cast<float*>(ws + L.w);
    t->g = reinterpret_cast<float*>(ws + L.g);
    t->m = reinterpret_cast<float*>(ws + L.m);
    t->v = reinterpret_cast<float*>(ws + L.v);
    t->wt = cfg->target_sync ? reinterpret_cast<float*>(ws + L.wt) : nullptr;
    t->wbt = cfg->target_sync && cfg->param_dtype == RP_BF16 ? reinterpret_cast<bf16_t*>(ws + L.wbt)
                                                              : nullptr;
    t->w2t = cfg->param_dtype == RP_F32 ? reinterpret_cast<float*>(ws + L.w2t) : nullptr;
    t->fused = !(cfg->flags & RP_TRAIN_LAYERED) && rp::fused_step_supported(*cfg, rp_);
    t->wide = !(cfg->flags & RP_TRAIN_LAYERED) && rp::wide_step_supported(*cfg, rp_);
    t->mid = !(cfg->flags & RP_TRAIN_LAYERED) && !t->fused && rp::mid_step_supported(*cfg, rp_);
    {
        auto at = [&](size_t off) { return reinterpret_cast<unsigned short*>(ws + off); };
        t->wd = rp::WideBuffers{at(L.W1T), at(L.W2b), at(L.W2T), at(L.W3T), at(L.W1Tt), at(L.W2Tt),
                                at(L.W3Tt), at(L.XT), at(L.H1T),
                                at(L.H2T), at(L.dQTh), at(L.dQTl), at(L.dZ2T), at(L.dZ1T),
                                reinterpret_cast<float*>(ws + L.part3),
                                reinterpret_cast<float*>(ws + L.part1),
                                reinterpret_cast<float*>(ws + L.part2)};
    }
    t->wb = cfg->param_dtype == RP_BF16 ? reinterpret_cast<bf16_t*>(ws + L.wb) : nullptr;
    t->X = ws + L.X;
    t->X_buf[0] = ws + L.X;
    t->X_buf[1] = ws + L.X2;
    t->gather_ahead = false;
    t->rec_skip_gather = false;
    t->rec_next = nullptr;
    t->rec_parity = 0;
    t->w_args_host[0] = t->w_args_host[1] = nullptr;
    t->act = reinterpret_cast<int*>(ws + L.act);
    t->rew = reinterpret_cast<float*>(ws + L.rew);
    t->term = ws + L.term;
    t->idx = reinterpret_cast<unsigned int*>(ws + L.idx);
    t->H1 = ws + L.H1;
    t->H2 = ws + L.H2;
    t->Q = reinterpret_cast<float*>(ws + L.Q);
    t->y = reinterpret_cast<float*>(ws + L.y);
    t->delta = reinterpret_cast<float*>(ws + L.delta);
    t->lossi = reinterpret_cast<float*>(ws + L.lossi);
    t->dQ = reinterpret_cast<float*>(ws + L.dQ);
    t->dZ2 = ws + L.dZ2;
    t->dZ1 = ws + L.dZ1;
    t->pre = reinterpret_cast<unsigned int*>(ws + L.pre);
    t->qpart = reinterpret_cast<float*>(ws + L.qpart);
    t->handoff = reinterpret_cast<unsigned long long*>(ws + L.handoff);
    t->ahead = reinterpret_cast<unsigned int*>(ws + L.ahead);
    t->qn_ahead = reinterpret_cast<float*>(ws + L.qn_ahead);
    t->epoch = 1;
    t->launch_seq = 0;
    t->handoff_ticks = rp::kHandoffTicks;
    t->handoff_break = false;
    t->graph = nullptr;
    t->graph_exec = nullptr;
    t->capture_stream = nullptr;
    t->host_step = 0;
    t->host_adam_t = 0;

    auto fail = [&](rp_status s) {
        train_destroy(t);
        return s;
    };
    hipError_t e = hipMemset(ws, 0, L.total);  // zero padding columns, moments, counters
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e != hipSuccess) {
        rp::set_error("train_create: clearing the workspace failed: %s", hipGetErrorString(e));
        return fail(RP_EHIP);
    }
    if (t->fused) {
        e = rp::fused_init();
        if (e != hipSuccess) {
            rp::set_error("train_create: allowing the row kernel's LDS size failed: %s", hipGetErrorString(e));
            return fail(RP_EHIP);
        }
    }
    if (t->wide) {
        e = rp::wide_init_buffers(t);
        if (e != hipSuccess) {
            rp::set_error("train_create: preparing the transposed buffers failed: %s", hipGetErrorString(e));
            return fail(RP_EHIP);
        }
    }
    rp_status s = train_set_state(t, host_init_params, nullptr, nullptr, 0, 0);
    if (s == RP_OK && t->wt) s = train_set_target(t, host_init_params);
    if (s != RP_OK) return fail(s);

    // pinned host slots for host-sourced payloads
    const size_t n_app = cfg->appends_per_step, sb = rp_->geom.state_bytes;
    t->pin_host = t->pin_dev = nullptr;
    t->pin_next = 0;
    for (auto& ev : t->pin_event) ev = nullptr;
    for (auto& live : t->pin_event_live) live = false;
    if (n_app) {
        size_t o = 0;
        auto take = [&](size_t bytes) { size_t at = o; o = rp::align_up(o + bytes, 16); return at; };
        take(n_app * sb);
        t->pin_off_s_next = take(n_app * sb);
        t->pin_off_a = take(n_app * 4);
        t->pin_off_r = take(n_app * 4);
        t->pin_off_term = take(n_app);
        t->pin_slot_bytes = rp::align_up(o, 128);
        void* hp = nullptr;
        void* dp = nullptr;
        e = hipHostMalloc(&hp, t->pin_slot_bytes * rp::kPinSlots, hipHostMallocMapped);
        if (e == hipSuccess) {
            t->pin_host = static_cast<unsigned char*>(hp);
            e = hipHostGetDevicePointer(&dp, hp, 0);
        }
        for (auto& ev : t->pin_event)
            if (e == hipSuccess) e = hipEventCreateWithFlags(&ev, hipEventDisableTiming);
        if (e != hipSuccess) {
            rp::set_error("train_create: pinned payload slots: %s", hipGetErrorString(e));
            return fail(RP_EHIP);
        }
        t->pin_dev = static_cast<unsigned char*>(dp);
    }
    t->payload_func = t->fused               ? rp::fused_rows_func(t->wt != nullptr, t->Dp, t->B)
                      : (t->wide || t->mid) ? rp::append_gather_func(rp_->geom)
                                            : rp::append_pair_func(rp_->geom);
    t->payload_kargs[0] = t->fused ? static_cast<void*>(&t->row_args) : static_cast<void*>(&t->append_args);
    t->payload_node[0] = nullptr;
    for (auto& run : t->runs) {
        run.graph = nullptr;
        run.exec = nullptr;
    }

    if (cfg->flags & RP_TRAIN_GRAPH) {
        // recorded once with the replay's staging area as a stand-in payload; the payload
        // kernel's argument is replaced before every launch
        const rp::Payload stand_in{rp_->stage_s, rp_->stage_s_next, rp_->stage_a, rp_->stage_r,
                                   rp_->stage_term};
        e = hipStreamCreateWithFlags(&t->capture_stream, hipStreamNonBlocking);
        t->gather_ahead = (t->mid || t->wide) && cfg->appends_per_step && rp_->cfg.sampling == RP_WITH_REPLACEMENT;
        if (t->wide) t->X_buf[1] = t->X_buf[0];   // (its optimizer kernel does not read the batch)
        if (e == hipSuccess) e = hipStreamBeginCapture(t->capture_stream, hipStreamCaptureModeThreadLocal);
        if (e == hipSuccess) {
            hipError_t ek = rp::enqueue_append_and_step(t, stand_in, t->capture_stream,
                                                        &t->kernels_per_step);
            e = hipStreamEndCapture(t->capture_stream, &t->graph);
            if (ek != hipSuccess) e = ek;
        }
        if (e == hipSuccess && rp::has_payload_node(t))
            e = rp::find_payload_nodes(t, t->graph, 1, t->payload_node, t->payload_np);
        if (e == hipSuccess) e = hipGraphInstantiate(&t->graph_exec, t->graph, nullptr, nullptr, 0);
        // the same for runs of several steps
        for (unsigned int g = 0; g < rp::kRuns && e == hipSuccess; ++g) {
            trainer::StepRun& run = t->runs[g];
            e = hipStreamBeginCapture(t->capture_stream, hipStreamCaptureModeThreadLocal);
            if (e != hipSuccess) break;
            hipError_t ek = hipSuccess;
            const unsigned int steps = rp::kRunSteps[g];
            for (unsigned int k = 0; k < steps && ek == hipSuccess; ++k) {
                rp::AppendGatherArgs next_gather;
                if (t->gather_ahead) {
                    // this step reads batch buffer k mod 2; all but the last also gather the
                    // next step's batch, into the other buffer, in their weights kernel's launch
                    t->X = t->X_buf[k & 1u];
                    t->rec_parity = k & 1u;
                    t->rec_skip_gather = k > 0;
                    if (k + 1 < steps) {
                        unsigned char* Xn = static_cast<unsigned char*>(t->X_buf[(k + 1) & 1u]);
                        next_gather = rp::make_append_gather_args(
                            rp_->geom, rp::RingPos{rp_->head, rp_->size, rp_->total}, cfg->appends_per_step,
                            stand_in, rp_->cfg.seed, nullptr, t->B,
                            rp::GatherOut{Xn, Xn + (size_t)t->B * t->Dp * t->elem, t->Dp, t->act, t->rew,
                                          t->term, t->idx, t->wide ? t->wd.XT : nullptr, t->Bp});
                        t->rec_next = &next_gather;
                    }
                }
                ek = rp::enqueue_append_and_step(t, stand_in, t->capture_stream, nullptr);
                t->rec_next = nullptr;
            }
            t->rec_skip_gather = false;
            t->rec_parity = 0;
            t->X = t->X_buf[0];
            e = hipStreamEndCapture(t->capture_stream, &run.graph);
            if (ek != hipSuccess) e = ek;
            if (e == hipSuccess && t->gather_ahead) {
                // node 0: the first step's append + gather kernel; node k > 0: step k - 1's weights kernel
                e = rp::find_payload_nodes(t, run.graph, 1, run.node, run.np);
                if (e == hipSuccess)
                    e = rp::find_kernel_nodes(t, run.graph, t->wide ? rp::opt_ahead_func() : rp::weights_ahead_func(t),
                                              steps - 1, run.node + 1, run.np + 1);
            } else if (e == hipSuccess && rp::has_payload_node(t))
                e = rp::find_payload_nodes(t, run.graph, rp::kRunSteps[g], run.node, run.np);
            if (e == hipSuccess) e = hipGraphInstantiate(&run.exec, run.graph, nullptr, nullptr, 0);
        }
        if (e != hipSuccess) {
            rp::set_error("train_create: recording the step graph failed: %s", hipGetErrorString(e));
            return fail(RP_EHIP);
        }
    } else {
        // the launch count is static
        // (a batch without duplicates is drawn by a kernel of its own wherever the step samples
        // through the replay's stand-alone gather)
        const bool own_draw = rp_->cfg.sampling == RP_DISTINCT && !t->fused &&
                              !((t->wide || t->mid) && cfg->appends_per_step);
        // the head's update is folded into the weights kernel when the action set fits one tile
        const bool folded_head = t->dueling && (t->fused || t->mid) && t->Ap == 32;
        t->kernels_per_step =
            (t->dueling && !folded_head ? 1u : 0u) + (own_draw ? 1u : 0u) +
            (t->fused ? 2u
             : t->mid ? rp::mid_step_kernels(t)
                      : (cfg->appends_per_step ? 1u : 0u) +
                            (t->wide ? (t->wt && cfg->batch % 128 ? 13u : 10u) : (t->wt ? 17u : 14u)));
    }
    *out = t;
    return RP_OK;
}

rp_status train_destroy(trainer_t* t) {
    if (!t) return RP_OK;
    if (t->graph_exec) (void)hipGraphExecDestroy(t->graph_exec);
    if (t->graph) (void)hipGraphDestroy(t->graph);
    for (auto& run : t->runs) {
        if (run.exec) (void)hipGraphExecDestroy(run.exec);
        if (run.graph) (void)hipGraphDestroy(run.graph);
    }
    if (t->capture_stream) (void)hipStreamDestroy(t->capture_stream);
    rp::free_weights_args(t);
    for (auto& ev : t->pin_event)
        if (ev) (void)hipEventDestroy(ev);
    if (t->pin_host) (void)hipHostFree(t->pin_host);
    delete t;
    return RP_OK;
}

rp_status train_step(trainer_t* t, const void* s, const void* s_next, const int32_t* a,
                     const float* r, const uint8_t* term, int src_is_device, void* hip_stream) {
    RP_REQUIRE(t, "train_step: null handle");
    replay* rpl = t->rp_;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const uint64_t n = t->cfg.appends_per_step;
    rp::Payload src{nullptr, nullptr, nullptr, nullptr, nullptr};
    const bool host_src = n && !src_is_device;
    if (n) {
        RP_REQUIRE(s && s_next && a && r && term, "train_step: null field array for the append");
        if (src_is_device)
            src = rp::Payload{static_cast<const unsigned char*>(s), static_cast<const unsigned char*>(s_next),
                              a, r, term};
        else
            RP_CHECK_HIP(rp::stage_host_payload(t, 0, n, s, s_next, a, r, term, &src));
    }
    const uint64_t total_after = rpl->total + n;
    const uint64_t size_after = rpl->size + n > rpl->cfg.capacity ? rpl->cfg.capacity : rpl->size + n;
    const bool train = total_after >= rpl->cfg.burn_in &&
                       size_after >= (rpl->cfg.sampling == RP_DISTINCT ? t->cfg.batch : 1u);
    if (!train) {
        if (n)
            RP_CHECK_HIP(rp::launch_append(rpl->geom, rp::RingPos{rpl->head, rpl->size, rpl->total}, n,
                                           src.s, src.s_next, src.a, src.r, src.term, st));
    } else if (t->graph_exec) {
        if (t->payload_node[0]) {
            rp::set_payload_args(t, src, 0);
            RP_CHECK_HIP(hipGraphExecKernelNodeSetParams(t->graph_exec, t->payload_node[0],
                                                         &t->payload_np[0]));
        }
        RP_CHECK_HIP(hipGraphLaunch(t->graph_exec, st));
    } else {
        RP_CHECK_HIP(rp::enqueue_append_and_step(t, src, st, nullptr));
    }
    if (host_src) RP_CHECK_HIP(rp::commit_host_slots(t, 1, st));
    rpl->total = total_after;
    rpl->size = size_after;
    rpl->head = (rpl->head + n) % rpl->cfg.capacity;
    if (!train) return RP_SKIPPED_BURN_IN;
    t->host_step += 1;
    t->host_adam_t += 1;
    return RP_OK;
}

rp_status train_step_batch(trainer_t* t, const void* s, const void* s_next, const int32_t* a,
                           const float* r, const uint8_t* term, void* hip_stream) {
    RP_REQUIRE(t, "train_step_batch: null handle");
    RP_REQUIRE(s && s_next && a && r && term, "train_step_batch: null field array");
    replay* rpl = t->rp_;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const rp::Payload batch{static_cast<const unsigned char*>(s),
                            static_cast<const unsigned char*>(s_next), a, r, term};
    if (t->fused && t->graph_exec && t->payload_node[0]) {
        // the recorded step with its row kernel pointed at the batch: nothing appended or drawn
        t->row_args.src = rp::Payload{nullptr, nullptr, nullptr, nullptr, nullptr};
        t->row_args.n_append = 0;
        t->row_args.batch = batch;
        t->row_args.from_batch = 1;
        t->row_args.head = rpl->head;
        t->row_args.step = t->host_step;
        t->row_args.size_after = (unsigned int)rpl->size;
        t->row_args.total_after = rpl->total;
        rp::set_adam_step(t->row_args, t->host_adam_t + 1, t->cfg.beta1, t->cfg.beta2);
        rp::stamp_launch(t, t->row_args);
        RP_CHECK_HIP(hipGraphExecKernelNodeSetParams(t->graph_exec, t->payload_node[0],
                                                     &t->payload_np[0]));
        RP_CHECK_HIP(hipGraphLaunch(t->graph_exec, st));
    } else {
        RP_CHECK_HIP(rp::enqueue_batch_step(t, batch, st));
    }
    t->host_step += 1;
    t->host_adam_t += 1;
    return RP_OK;
}

rp_status train_steps(trainer_t* t, uint64_t count, const void* s, const void* s_next,
                      const int32_t* a, const float* r, const uint8_t* term, int src_is_device,
                      void* hip_stream, uint64_t* executed) {
    RP_REQUIRE(t, "train_steps: null handle");
    replay* rpl = t->rp_;
    const uint64_t n = t->cfg.appends_per_step;
    const size_t sb = rpl->geom.state_bytes;
    RP_REQUIRE(n == 0 || (s && s_next && a && r && term), "train_steps: null field array for the append");
    uint64_t done = 0;
    for (uint64_t k = 0; k < count;) {
        const uint64_t o = k * n;
        // several steps in one graph launch when all of them train (new experiences in host
        // memory go through one pinned slot per step)
        const bool host_src = n && !src_is_device;
        // What is left is made in recorded runs, the short ones first: the longest run (the
        // longest the staging area takes, for host arrays) as often as it fits, and before
        // those the powers of two that make up the rest, smallest first.  The GPU then starts
        // on a call's first steps after few nodes' arguments have been replaced, and the long
        // runs are prepared while it works.
        const uint64_t longest = host_src ? rp::kRunStepsHostPayload : rp::kRunStepsMax;
        const uint64_t rest = (count - k) % longest;
        const uint64_t want = rest ? (rest & (~rest + 1)) : longest;
        trainer::StepRun* run = nullptr;
        uint64_t K = 0;
        for (unsigned int g = 0; g < rp::kRuns && !run; ++g) {
            const uint64_t steps = rp::kRunSteps[g];
            if (t->runs[g].exec && steps <= want) {
                run = &t->runs[g];
                K = steps;
            }
        }
        hipGraphExec_t const run_exec = run ? run->exec : nullptr;
        hipGraphNode_t* const run_node = run ? run->node : nullptr;
        hipKernelNodeParams* const run_np = run ? run->np : nullptr;
        if (run_exec && (!host_src || rp::has_payload_node(t)) &&
            rpl->total + n >= rpl->cfg.burn_in &&
            rpl->size + n >= (rpl->cfg.sampling == RP_DISTINCT ? t->cfg.batch : 1u)) {
            for (unsigned int j = 0; j < K && rp::has_payload_node(t); ++j) {
                const uint64_t oj = o + j * n;
                rp::Payload src =
                    n ? rp::Payload{static_cast<const unsigned char*>(s) + oj * sb,
                                    static_cast<const unsigned char*>(s_next) + oj * sb, a + oj, r + oj,
                                    term + oj}
                      : rp::Payload{nullptr, nullptr, nullptr, nullptr, nullptr};
                if (host_src)
                    RP_CHECK_HIP(rp::stage_host_payload(t, j, n, src.s, src.s_next, src.a, src.r, src.term, &src));
                rp::set_payload_args(t, src, j);
                if (t->gather_ahead && j && t->wide)
                    RP_CHECK_HIP(rp::patch_opt_ahead_node(t, run_exec, run_node[j], run_np[j], t->append_args));
                else if (t->gather_ahead && j)
                    RP_CHECK_HIP(rp::patch_weights_ahead_node(t, run_exec, run_node[j], run_np[j], (j - 1u) & 1u,
                                                              t->append_args));
                else
                    RP_CHECK_HIP(hipGraphExecKernelNodeSetParams(run_exec, run_node[j], &run_np[j]));
            }
            RP_CHECK_HIP(hipGraphLaunch(run_exec, static_cast<hipStream_t>(hip_stream)));
            if (host_src)
                RP_CHECK_HIP(rp::commit_host_slots(t, (unsigned int)K, static_cast<hipStream_t>(hip_stream)));
            const uint64_t cap = rpl->cfg.capacity;
            rpl->total += K * n;
            rpl->size = rpl->size + K * n > cap ? cap : rpl->size + K * n;
            rpl->head = (rpl->head + K * n) % cap;
            t->host_step += K;
            t->host_adam_t += K;
            done += K;
            k += K;
            continue;
        }
        const rp_status st =
            n ? train_step(t, static_cast<const unsigned char*>(s) + o * sb,
                           static_cast<const unsigned char*>(s_next) + o * sb, a + o, r + o,
                           term + o, src_is_device, hip_stream)
              : train_step(t, nullptr, nullptr, nullptr, nullptr, nullptr, 0, hip_stream);
        if (st < 0) {
            if (executed) *executed = done;
            return st;
        }
        done += st == RP_OK;
        ++k;
    }
    if (executed) *executed = done;
    return RP_OK;
}

rp_status train_get_params(trainer_t* t, float* params) {
    RP_REQUIRE(t && params, "train_get_params: null argument");
    std::vector<float> pad(t->n_dev);
    RP_CHECK_HIP(hipDeviceSynchronize());
    RP_CHECK_HIP(hipMemcpy(pad.data(), t->w, t->n_dev * 4, hipMemcpyDeviceToHost));
    rp::unpad_params(t, pad, params);
    return RP_OK;
}

rp_status train_get_target(trainer_t* t, float* params) {
    RP_REQUIRE(t && params, "train_get_target: null argument");
    std::vector<float> pad(t->n_dev);
    RP_CHECK_HIP(hipDeviceSynchronize());
    RP_CHECK_HIP(hipMemcpy(pad.data(), t->wt ? t->wt : t->w, t->n_dev * 4, hipMemcpyDeviceToHost));
    rp::unpad_params(t, pad, params);
    return RP_OK;
}

rp_status train_set_target(trainer_t* t, const float* params) {
    RP_REQUIRE(t && params, "train_set_target: null argument");
    RP_REQUIRE(t->wt, "train_set_target: this trainer has no target network (target_sync = 0)");
    if (++t->epoch == 0) ++t->epoch;   // target values computed a step ahead no longer hold
    std::vector<float> pad;
    RP_CHECK_HIP(hipDeviceSynchronize());
    rp::pad_params(t, params, pad);
    RP_CHECK_HIP(hipMemcpy(t->wt, pad.data(), t->n_dev * 4, hipMemcpyHostToDevice));
    if (t->wide) RP_CHECK_HIP(rp::wide_set_weights(t, pad.data(), true));
    if (t->wbt) {
        hipLaunchKernelGGL(rp::to_bf16_kernel, dim3((t->n_padded + rp::kThreads - 1) / rp::kThreads),
                           dim3(rp::kThreads), 0, nullptr, (unsigned int)t->n_padded, t->wt, t->wbt);
        RP_CHECK_HIP(hipGetLastError());
    }
    RP_CHECK_HIP(hipDeviceSynchronize());
    return RP_OK;
}

rp_status train_get_grads(trainer_t* t, float* grads) {
    RP_REQUIRE(t && grads, "train_get_grads: null argument");
    std::vector<float> pad(t->n_dev);
    RP_CHECK_HIP(hipDeviceSynchronize());
    RP_CHECK_HIP(hipMemcpy(pad.data(), t->g, t->n_dev * 4, hipMemcpyDeviceToHost));
    rp::unpad_params(t, pad, grads);
    return RP_OK;
}

rp_status train_get_opt_state(trainer_t* t, float* m, float* v, uint64_t* adam_t, uint64_t* step) {
    RP_REQUIRE(t, "train_get_opt_state: null handle");
    std::vector<float> pad(t->n_dev);
    RP_CHECK_HIP(hipDeviceSynchronize());
    if (m) {
        RP_CHECK_HIP(hipMemcpy(pad.data(), t->m, t->n_dev * 4, hipMemcpyDeviceToHost));
        rp::unpad_params(t, pad, m);
    }
    if (v) {
        RP_CHECK_HIP(hipMemcpy(pad.data(), t->v, t->n_dev * 4, hipMemcpyDeviceToHost));
        rp::unpad_params(t, pad, v);
    }
    TrainCounters c;
    RP_CHECK_HIP(hipMemcpy(&c, t->ctr, sizeof(c), hipMemcpyDeviceToHost));
    if (adam_t) *adam_t = c.adam_t;
    if (step) *step = c.step;
    RP_REQUIRE_STATE(!c.handoff_missed, "train_get_opt_state: a train step's workgroups missed a hand-over");
    return RP_OK;
}

rp_status train_set_state(trainer_t* t, const float* params, const float* m, const float* v,
                          uint64_t adam_t, uint64_t step) {
    RP_REQUIRE(t && params, "train_set_state: null argument");
    if (++t->epoch == 0) ++t->epoch;
    std::vector<float> pad;
    RP_CHECK_HIP(hipDeviceSynchronize());
    rp::pad_params(t, params, pad);
    RP_CHECK_HIP(hipMemcpy(t->w, pad.data(), t->n_dev * 4, hipMemcpyHostToDevice));
    if (t->wide) RP_CHECK_HIP(rp::wide_set_weights(t, pad.data(), false));
    if (t->w2t) {
        const size_t H = t->H, G = t->Hb;
        std::vector<float> tr(G * H);
        for (size_t j = 0; j < H; ++j)
            for (size_t k = 0; k < G; ++k) tr[k * H + j] = pad[t->oW2 + j * G + k];
        RP_CHECK_HIP(hipMemcpy(t->w2t, tr.data(), G * H * 4, hipMemcpyHostToDevice));
    }
    if (m) {
        rp::pad_params(t, m, pad, false);
        RP_CHECK_HIP(hipMemcpy(t->m, pad.data(), t->n_dev * 4, hipMemcpyHostToDevice));
    }
    if (v) {
        rp::pad_params(t, v, pad, false);
        RP_CHECK_HIP(hipMemcpy(t->v, pad.data(), t->n_dev * 4, hipMemcpyHostToDevice));
    }
    TrainCounters c;
    RP_CHECK_HIP(hipMemcpy(&c, t->ctr, sizeof(c), hipMemcpyDeviceToHost));
    c.adam_t = adam_t;
    c.step = step;
    c.handoff_missed = 0;
    c.pw1 = std::pow((double)t->cfg.beta1, (double)adam_t);
    c.pw2 = std::pow((double)t->cfg.beta2, (double)adam_t);
    RP_CHECK_HIP(hipMemcpy(t->ctr, &c, sizeof(c), hipMemcpyHostToDevice));
    t->host_step = step;
    t->host_adam_t = adam_t;
    if (t->wb) {
        hipLaunchKernelGGL(rp::to_bf16_kernel, dim3((t->n_padded + rp::kThreads - 1) / rp::kThreads),
                           dim3(rp::kThreads), 0, nullptr, (unsigned int)t->n_padded, t->w, t->wb);
        RP_CHECK_HIP(hipGetLastError());
    }
    RP_CHECK_HIP(hipDeviceSynchronize());
    return RP_OK;
}

rp_status train_get_last(trainer_t* t, float* q, float* q_next, float* y, float* delta, float* loss,
                         uint32_t* idx) {
    RP_REQUIRE(t, "train_get_last: null handle");
    const size_t B = t->B, A = t->cfg.num_actions, Ap = t->Ap;
    RP_CHECK_HIP(hipDeviceSynchronize());
    if (q || q_next) {
        std::vector<float> Q(2 * B * Ap);
        RP_CHECK_HIP(hipMemcpy(Q.data(), t->Q, Q.size() * 4, hipMemcpyDeviceToHost));
        for (size_t i = 0; i < B; ++i) {
            if (q) memcpy(q + i * A, &Q[i * Ap], A * 4);
            if (q_next) memcpy(q_next + i * A, &Q[(B + i) * Ap], A * 4);
        }
    }
    if (y) RP_CHECK_HIP(hipMemcpy(y, t->y, B * 4, hipMemcpyDeviceToHost));
    if (delta) RP_CHECK_HIP(hipMemcpy(delta, t->delta, B * 4, hipMemcpyDeviceToHost));
    if (idx) RP_CHECK_HIP(hipMemcpy(idx, t->idx, B * 4, hipMemcpyDeviceToHost));
    TrainCounters c;
    RP_CHECK_HIP(hipMemcpy(&c, t->ctr, sizeof(c), hipMemcpyDeviceToHost));
    if (loss) *loss = c.loss;
    RP_REQUIRE_STATE(!c.handoff_missed, "train_get_last: a train step's workgroups missed a hand-over");
    return RP_OK;
}

rp_status train_set_handoff_wait(trainer_t* t, uint64_t ticks, int break_pairing) {
    RP_REQUIRE(t, "train_set_handoff_wait: null handle");
    RP_REQUIRE(ticks <= (uint64_t)1 << 40, "train_set_handoff_wait: limit beyond 2^40 ticks");
    t->handoff_ticks = ticks ? (long long)ticks : rp::kHandoffTicks;
    t->handoff_break = break_pairing != 0;
    return RP_OK;
}

rp_status train_get_target_source(trainer_t* t, uint32_t* from_table) {
    RP_REQUIRE(t && from_table, "train_get_target_source: null argument");
    RP_CHECK_HIP(hipDeviceSynchronize());
    TrainCounters c;
    RP_CHECK_HIP(hipMemcpy(&c, t->ctr, sizeof(c), hipMemcpyDeviceToHost));
    *from_table = c.from_table;
    return RP_OK;
}

rp_status train_kernels_per_step(trainer_t* t, uint32_t* n) {
    RP_REQUIRE(t && n, "train_kernels_per_step: null argument");
    *n = t->kernels_per_step;
    return RP_OK;
}

}  // extern "C"
