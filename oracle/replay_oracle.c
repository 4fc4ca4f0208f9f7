/*
 * CPU oracle for the device-resident experience-replay train step.
 * TEST INFRASTRUCTURE ONLY: see replay_oracle.h.  Plain scalar C; the only
 * concession to speed is an OpenMP "parallel for" over loops whose iterations
 * are independent, which leaves every sum in the same order as the serial code.
 */
#include "replay_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static int g_threads = 1;

void oracle_set_threads(int n) {
    g_threads = n < 1 ? 1 : n;
#ifdef _OPENMP
    omp_set_num_threads(g_threads);
#endif
}
int oracle_get_threads(void) {
#ifdef _OPENMP
    return g_threads;
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------------
 * Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as
 * easy as 1, 2, 3", SC'11).  Ten rounds; the key is advanced by the Weyl
 * constants between rounds.
 * --------------------------------------------------------------------- */
void oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
    const uint64_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
    const uint32_t W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        if (round > 0) {
            k0 += W0;
            k1 += W1;
        }
        uint64_t p0 = M0 * (uint64_t)c0;
        uint64_t p1 = M1 * (uint64_t)c2;
        uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0;
        uint32_t hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
        uint32_t n0 = hi1 ^ c1 ^ k0;
        uint32_t n1 = lo1;
        uint32_t n2 = hi0 ^ c3 ^ k1;
        uint32_t n3 = lo0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/*
 * Uniform integer in [0, n_choices) for draw i of sampling step `step`
 * (Methods: integers drawn uniformly between 0 and the current replay size,
 * with replacement).  The generator is keyed by the seed; the counter holds
 * (i div 4, stream 0, step); draw i takes word i mod 4 of that block; the
 * 32-bit word x is mapped to floor(x * n_choices / 2^32).
 */
uint32_t oracle_uniform_index(uint64_t seed, uint64_t step, uint32_t i, uint64_t n_choices) {
    uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    uint32_t ctr[4] = {i / 4u, 0u, (uint32_t)step, (uint32_t)(step >> 32)};
    uint32_t x[4];
    oracle_philox4x32_10(ctr, key, x);
    return (uint32_t)(((uint64_t)x[i % 4u] * n_choices) >> 32);
}

/*
 * Member i (i < n) of a sample of distinct integers from [0, n)  (Methods: the in-RAM replay
 * samples without duplicates; the author wants the device replay to do so too).
 * The sample is the image of 0, 1, 2, ... under a keyed permutation of [0, n), so its members
 * are distinct by construction and each is a pure function of (seed, step, i).  The permutation
 * is a swap-or-not shuffle (Hoang, Morris, Rogaway, CRYPTO 2012), which works on a domain of any
 * size: in round r every x is paired with its partner K_r - x (mod n) and the pair is swapped
 * or not according to one pseudorandom bit that both members agree on (it is a function of the
 * larger of the two).  Rounds: 2 * bitlen(n - 1) + 8.  Randomness comes from Philox4x32-10 with
 * key = seed: K_r = floor(w * n / 2^32) with w = word r mod 4 of counter (r div 4, 1, step);
 * the bit of round r for pair maximum m = bit 0 of word 0 of counter (m, 2 + r, step).
 */
uint32_t oracle_distinct_index(uint64_t seed, uint64_t step, uint32_t i, uint64_t n) {
    uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    unsigned bitlen = 0;
    for (uint64_t v = n - 1; v; v >>= 1) ++bitlen;
    const uint32_t rounds = 2 * bitlen + 8;
    uint64_t x = i;
    for (uint32_t r = 0; r < rounds; ++r) {
        uint32_t kc[4] = {r / 4u, 1u, (uint32_t)step, (uint32_t)(step >> 32)}, kw[4];
        oracle_philox4x32_10(kc, key, kw);
        uint64_t K = ((uint64_t)kw[r % 4u] * n) >> 32;
        uint64_t partner = (K + n - x) % n;
        uint64_t m = partner > x ? partner : x;
        uint32_t bc[4] = {(uint32_t)m, 2u + r, (uint32_t)step, (uint32_t)(step >> 32)}, bw[4];
        oracle_philox4x32_10(bc, key, bw);
        if (bw[0] & 1u) x = partner;
    }
    return (uint32_t)x;
}

void oracle_uniform_indices(uint64_t seed, uint64_t step0, uint64_t nsteps, uint32_t batch,
                            uint64_t n_choices, uint32_t* out) {
    for (uint64_t k = 0; k < nsteps; ++k)
        for (uint32_t i = 0; i < batch; ++i)
            out[k * batch + i] = oracle_uniform_index(seed, step0 + k, i, n_choices);
}

/* ------------------------------------------------------------------------
 * FIFO ring (Related Work: fixed size, starts empty, newest replace oldest
 * first-in first-out; Methods: add / sample API).  The k-th experience ever
 * added (k from 0) lives in slot k mod capacity.
 * --------------------------------------------------------------------- */
struct oracle_ring {
    uint64_t capacity, head, size, total, burn_in;
    uint32_t state_dim, state_dtype, layout;
    size_t   state_bytes; /* bytes of one stored state */
    uint8_t* s;           /* [capacity][state_bytes] old states          */
    uint8_t* s_next;      /* [capacity][state_bytes] new states (PAIR)   */
    int32_t* a;
    float*   r;
    uint8_t* term;
};

static size_t elem_bytes(uint32_t dtype) {
    return dtype == ORACLE_F32 ? 4 : dtype == ORACLE_BF16 ? 2 : 1;
}

oracle_ring* oracle_ring_create(uint64_t capacity, uint32_t state_dim, uint32_t state_dtype,
                                uint32_t layout, uint64_t burn_in) {
    if (capacity == 0 || state_dim == 0 || state_dtype > ORACLE_U8 || layout > ORACLE_CHAIN)
        return NULL;
    oracle_ring* g = (oracle_ring*)calloc(1, sizeof(*g));
    if (!g) return NULL;
    g->capacity = capacity;
    g->burn_in = burn_in;
    g->state_dim = state_dim;
    g->state_dtype = state_dtype;
    g->layout = layout;
    g->state_bytes = (size_t)state_dim * elem_bytes(state_dtype);
    g->s = (uint8_t*)calloc(capacity, g->state_bytes);
    g->s_next = layout == ORACLE_PAIR ? (uint8_t*)calloc(capacity, g->state_bytes) : NULL;
    g->a = (int32_t*)calloc(capacity, sizeof(int32_t));
    g->r = (float*)calloc(capacity, sizeof(float));
    g->term = (uint8_t*)calloc(capacity, 1);
    if (!g->s || (layout == ORACLE_PAIR && !g->s_next) || !g->a || !g->r || !g->term) {
        oracle_ring_destroy(g);
        return NULL;
    }
    return g;
}

void oracle_ring_destroy(oracle_ring* g) {
    if (!g) return;
    free(g->s); free(g->s_next); free(g->a); free(g->r); free(g->term);
    free(g);
}

int oracle_ring_append(oracle_ring* g, uint64_t n, const void* s, const void* s_next,
                       const int32_t* a, const float* r, const uint8_t* term) {
    if (!g || n > g->capacity) return -1;
    if (n == 0) return 0;
    if (!s || !a || !r || !term || (g->layout == ORACLE_PAIR && !s_next)) return -1;
    for (uint64_t k = 0; k < n; ++k) {
        uint64_t slot = g->total % g->capacity;
        memcpy(g->s + slot * g->state_bytes, (const uint8_t*)s + k * g->state_bytes,
               g->state_bytes);
        if (g->layout == ORACLE_PAIR)
            memcpy(g->s_next + slot * g->state_bytes,
                   (const uint8_t*)s_next + k * g->state_bytes, g->state_bytes);
        g->a[slot] = a[k];
        g->r[slot] = r[k];
        g->term[slot] = term[k] ? 1 : 0;
        g->total += 1;
        if (g->size < g->capacity) g->size += 1;
        g->head = g->total % g->capacity;
    }
    return 0;
}

void oracle_ring_state(const oracle_ring* g, uint64_t* head, uint64_t* size, uint64_t* total) {
    if (head) *head = g->head;
    if (size) *size = g->size;
    if (total) *total = g->total;
}

int oracle_ring_read(const oracle_ring* g, uint64_t first_slot, uint64_t n, void* s, void* s_next,
                     int32_t* a, float* r, uint8_t* term) {
    if (!g || first_slot >= g->capacity || n > g->capacity) return -1;
    for (uint64_t k = 0; k < n; ++k) {
        uint64_t slot = (first_slot + k) % g->capacity;
        if (s) memcpy((uint8_t*)s + k * g->state_bytes, g->s + slot * g->state_bytes,
                      g->state_bytes);
        if (s_next && g->layout == ORACLE_PAIR)
            memcpy((uint8_t*)s_next + k * g->state_bytes, g->s_next + slot * g->state_bytes,
                   g->state_bytes);
        if (a) a[k] = g->a[slot];
        if (r) r[k] = g->r[slot];
        if (term) term[k] = g->term[slot];
    }
    return 0;
}

/*
 * One sample of `batch` slot numbers.  No sampling before burn-in completes
 * (Related Work: training is skipped during burn-in).  PAIR: uniform over the
 * `size` filled slots, which are slots 0..size-1.  CHAIN: the newest slot has
 * no successor yet, so the draw is over the size-1 older experiences, counted
 * from the oldest one.
 */
int oracle_ring_sample_mode(const oracle_ring* g, uint64_t seed, uint64_t step, uint32_t batch,
                            int distinct, uint32_t* idx) {
    if (!g || !idx || batch == 0) return -1;
    if (g->total < g->burn_in) return 1;
    /* experiences that can be drawn; a sample of distinct ones needs at least `batch` of them */
    uint64_t choices = g->layout == ORACLE_PAIR ? g->size : (g->size < 2 ? 0 : g->size - 1);
    if (choices == 0 || (distinct && choices < batch)) return 1;
    uint64_t oldest = (g->head + g->capacity - g->size) % g->capacity;
    for (uint32_t i = 0; i < batch; ++i) {
        uint64_t u = distinct ? oracle_distinct_index(seed, step, i, choices)
                              : oracle_uniform_index(seed, step, i, choices);
        idx[i] = g->layout == ORACLE_PAIR ? (uint32_t)u : (uint32_t)((oldest + u) % g->capacity);
    }
    return 0;
}

int oracle_ring_sample(const oracle_ring* g, uint64_t seed, uint64_t step, uint32_t batch,
                       uint32_t* idx) {
    return oracle_ring_sample_mode(g, seed, step, batch, 0, idx);
}

/* one state out of the ring into a batch row: raw bits, or u8 / 255 as float */
static void emit_state(const oracle_ring* g, const uint8_t* src, void* out, uint32_t row) {
    if (g->state_dtype == ORACLE_U8) {
        float* dst = (float*)out + (size_t)row * g->state_dim;
        for (uint32_t d = 0; d < g->state_dim; ++d) dst[d] = (float)src[d] / 255.0f;
    } else {
        memcpy((uint8_t*)out + (size_t)row * g->state_bytes, src, g->state_bytes);
    }
}

int oracle_ring_gather(const oracle_ring* g, const uint32_t* idx, uint32_t batch, void* out_s,
                       void* out_s_next, int32_t* out_a, float* out_r, uint8_t* out_term) {
    if (!g || !idx) return -1;
    for (uint32_t i = 0; i < batch; ++i) {
        uint64_t p = idx[i];
        if (p >= g->capacity) return -1;
        if (out_s) emit_state(g, g->s + p * g->state_bytes, out_s, i);
        if (out_s_next) {
            const uint8_t* nxt = g->layout == ORACLE_PAIR
                                     ? g->s_next + p * g->state_bytes
                                     : g->s + ((p + 1) % g->capacity) * g->state_bytes;
            emit_state(g, nxt, out_s_next, i);
        }
        if (out_a) out_a[i] = g->a[p];
        if (out_r) out_r[i] = g->r[p];
        if (out_term) out_term[i] = g->term[p];
    }
    return 0;
}

/* ------------------------------------------------------------------------
 * bfloat16: the upper 16 bits of an IEEE binary32, round to nearest even.
 * --------------------------------------------------------------------- */
uint16_t oracle_bf16_bits(float x) {
    uint32_t u;
    memcpy(&u, &x, 4);
    if ((u & 0x7F800000u) == 0x7F800000u && (u & 0x007FFFFFu)) /* NaN stays NaN */
        return (uint16_t)((u >> 16) | 0x0040u);
    uint32_t lower = u & 0xFFFFu, upper = u >> 16;
    if (lower > 0x8000u || (lower == 0x8000u && (upper & 1u))) upper += 1;
    return (uint16_t)upper;
}

double oracle_round_bf16(double x) {
    uint32_t u = (uint32_t)oracle_bf16_bits((float)x) << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

/* ------------------------------------------------------------------------
 * Q-network: D -> H -> G -> A, ReLU after the two hidden layers, linear out
 * (G = cfg->hidden2, or H when that is 0).
 *
 * With cfg->dueling the last layer is the dueling head of the paper (Deep
 * Q-Network Model: one shared layer, then a value stream and an advantage
 * stream, 128 and 2 x 512 units in the paper, i.e. H = 128, G = 1024): the
 * second hidden layer is the two streams side by side, units 0 .. G/2-1 feed a
 * scalar state value V and units G/2 .. G-1 feed one advantage per action, and
 *     Q(s, a) = V(s) + A(s, a) - mean_a' A(s, a').
 * The last layer then has 1 + A outputs (column 0 = V, column 1 + a = A(., a));
 * its weights from the other stream's units are structurally zero and get no
 * gradient.
 * --------------------------------------------------------------------- */
static uint32_t out_width(const oracle_train_cfg* cfg) {
    return cfg->num_actions + (cfg->dueling ? 1u : 0u);
}
/* width of the second hidden layer (hidden2 = 0: as wide as the first) */
static uint32_t width2(const oracle_train_cfg* cfg) {
    return cfg->hidden2 ? cfg->hidden2 : cfg->hidden;
}

size_t oracle_param_count2(uint32_t D, uint32_t H, uint32_t G, uint32_t A) {
    return (size_t)D * H + H + (size_t)H * G + G + (size_t)G * A + A;
}
size_t oracle_param_count(uint32_t D, uint32_t H, uint32_t A) {
    return oracle_param_count2(D, H, H, A);
}

typedef struct {
    const double *W1, *b1, *W2, *b2, *W3, *b3;
} net_view;

static net_view view_params(const double* p, uint32_t D, uint32_t H, uint32_t G, uint32_t A) {
    net_view n;
    n.W1 = p;               p += (size_t)D * H;
    n.b1 = p;               p += H;
    n.W2 = p;               p += (size_t)H * G;
    n.b2 = p;               p += G;
    n.W3 = p;               p += (size_t)G * A;
    n.b3 = p;
    (void)A;
    return n;
}

/* 1 where the dueling head has a weight from unit k of the second hidden layer to output o */
static int head_connected(const oracle_train_cfg* cfg, uint32_t k, uint32_t o) {
    if (!cfg->dueling) return 1;
    const int value_stream = k < width2(cfg) / 2;
    return o == 0 ? value_stream : !value_stream;
}

/* the weights the matrix products see: bf16-rounded copies in mixed precision, and the
 * structural zeros of the dueling head */
static double* effective_params(const oracle_train_cfg* cfg, const double* params) {
    const uint32_t D = cfg->state_dim, H = cfg->hidden, G = width2(cfg), O = out_width(cfg);
    size_t n = oracle_param_count2(D, H, G, O);
    double* e = (double*)malloc(n * sizeof(double));
    memcpy(e, params, n * sizeof(double));
    size_t oW1 = 0, oW2 = (size_t)D * H + H, oW3 = oW2 + (size_t)H * G + G;
    if (cfg->bf16) {
        for (size_t k = 0; k < (size_t)D * H; ++k) e[oW1 + k] = oracle_round_bf16(e[oW1 + k]);
        for (size_t k = 0; k < (size_t)H * G; ++k) e[oW2 + k] = oracle_round_bf16(e[oW2 + k]);
        for (size_t k = 0; k < (size_t)G * O; ++k) e[oW3 + k] = oracle_round_bf16(e[oW3 + k]);
    }
    for (uint32_t k = 0; k < G; ++k)
        for (uint32_t o = 0; o < O; ++o)
            if (!head_connected(cfg, k, o)) e[oW3 + (size_t)k * O + o] = 0.0;
    return e;
}

/* out[i][o] = act(sum_k in[i][k] * W[k][o] + b[o]) */
static void dense(const double* in, uint32_t n, uint32_t K, const double* W, const double* b,
                  uint32_t O, int relu, int round_bf16, double* out) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < (int64_t)n; ++i) {
        for (uint32_t o = 0; o < O; ++o) {
            double acc = 0.0;
            for (uint32_t k = 0; k < K; ++k) acc += in[(size_t)i * K + k] * W[(size_t)k * O + o];
            acc += b[o];
            if (relu && !(acc > 0.0)) acc = 0.0;
            if (round_bf16) acc = oracle_round_bf16(acc);
            out[(size_t)i * O + o] = acc;
        }
    }
}

/* Q[i][a] from the last layer's outputs z[i][.]: the outputs themselves, or the dueling combine */
static void head_combine(const oracle_train_cfg* cfg, const double* z, uint32_t n, double* Q) {
    const uint32_t A = cfg->num_actions, O = out_width(cfg);
    for (uint32_t i = 0; i < n; ++i) {
        if (!cfg->dueling) {
            for (uint32_t a = 0; a < A; ++a) Q[(size_t)i * A + a] = z[(size_t)i * O + a];
            continue;
        }
        double mean = 0.0;
        for (uint32_t a = 0; a < A; ++a) mean += z[(size_t)i * O + 1 + a];
        mean /= A;
        for (uint32_t a = 0; a < A; ++a)
            Q[(size_t)i * A + a] = z[(size_t)i * O] + z[(size_t)i * O + 1 + a] - mean;
    }
}

static void forward_with(const oracle_train_cfg* cfg, const double* eff, const double* X,
                         uint32_t n, double* h1, double* h2, double* Q) {
    const uint32_t D = cfg->state_dim, H = cfg->hidden, G = width2(cfg), O = out_width(cfg);
    net_view w = view_params(eff, D, H, G, O);
    double* t1 = h1 ? h1 : (double*)malloc((size_t)n * H * sizeof(double));
    double* t2 = h2 ? h2 : (double*)malloc((size_t)n * G * sizeof(double));
    double* z = (double*)malloc((size_t)n * O * sizeof(double));
    dense(X, n, D, w.W1, w.b1, H, 1, (int)cfg->bf16, t1);
    dense(t1, n, H, w.W2, w.b2, G, 1, (int)cfg->bf16, t2);
    dense(t2, n, G, w.W3, w.b3, O, 0, 0, z);
    head_combine(cfg, z, n, Q);
    free(z);
    if (!h1) free(t1);
    if (!h2) free(t2);
}

void oracle_mlp_forward(const oracle_train_cfg* cfg, const double* params, const double* X,
                        uint32_t n, double* h1, double* h2, double* Q) {
    double* eff = effective_params(cfg, params);
    forward_with(cfg, eff, X, n, h1, h2, Q);
    free(eff);
}

/* per-sample loss of the TD error d: half square, or Huber with threshold 1 */
static double sample_loss(uint32_t kind, double d) {
    if (kind == ORACLE_MSE) return 0.5 * d * d;
    return fabs(d) <= 1.0 ? 0.5 * d * d : fabs(d) - 0.5;
}
/* its derivative with respect to d */
static double sample_loss_slope(uint32_t kind, double d) {
    if (kind == ORACLE_MSE) return d;
    return d > 1.0 ? 1.0 : d < -1.0 ? -1.0 : d;
}

double oracle_loss_fixed_targets(const oracle_train_cfg* cfg, const double* params,
                                 const double* S, const int32_t* a, const double* y) {
    const uint32_t A = cfg->num_actions, B = cfg->batch;
    double* Q = (double*)malloc((size_t)B * A * sizeof(double));
    oracle_mlp_forward(cfg, params, S, B, NULL, NULL, Q);
    double L = 0.0;
    for (uint32_t i = 0; i < B; ++i) L += sample_loss(cfg->loss, y[i] - Q[(size_t)i * A + a[i]]);
    free(Q);
    return L / B;
}

/*
 * The parameter update of one step from a given gradient g of the mean loss (Deep Q-Network
 * Model: the update equation moves w against the gradient, scaled by the step size alpha).
 * SGD: w <- w - lr g.  Adam (Kingma & Ba): t <- t + 1, m <- beta1 m + (1 - beta1) g,
 * v <- beta2 v + (1 - beta2) g^2, w <- w - lr (m / (1 - beta1^t)) / (sqrt(v / (1 - beta2^t)) + eps).
 * m, v, t are untouched by SGD (and may be NULL then).
 */
void oracle_opt_apply(const oracle_train_cfg* cfg, size_t n, double* params, double* m, double* v,
                      uint64_t* t, const double* g) {
    if (cfg->opt == ORACLE_SGD) {
        for (size_t k = 0; k < n; ++k) params[k] -= cfg->lr * g[k];
        return;
    }
    *t += 1;
    double c1 = 1.0 - pow(cfg->beta1, (double)*t);
    double c2 = 1.0 - pow(cfg->beta2, (double)*t);
    for (size_t k = 0; k < n; ++k) {
        m[k] = cfg->beta1 * m[k] + (1.0 - cfg->beta1) * g[k];
        v[k] = cfg->beta2 * v[k] + (1.0 - cfg->beta2) * g[k] * g[k];
        params[k] -= cfg->lr * (m[k] / c1) / (sqrt(v[k] / c2) + cfg->eps);
    }
}

/*
 * One Q-learning step (Deep Q-Network Model, the update equation; Integration:
 * Q(s,a) is entry i*A + a_i of the flattened network output).
 *   y_i     = r_i + gamma * (1 - terminal_i) * max_a' Q_w(s'_i, a')   (a constant)
 *   delta_i = y_i - Q_w(s_i, a_i)
 *   L       = mean_i loss(delta_i)
 * followed by plain backpropagation of L through Q_w(s_i, .) only and an SGD
 * or Adam update.
 */
/*
 * target_params (may be NULL): parameters of the frozen target network (Deep
 * Q-Network Model: a non-trainable copy of the weights gives the target, and is
 * overwritten with the trained weights every fixed number of steps); Q(s', .)
 * is then evaluated with it.  NULL = the trained network itself, which is the
 * update equation as printed (one w on both sides).
 */
void oracle_train_step_target(const oracle_train_cfg* cfg, double* params,
                              const double* target_params, double* m, double* v, uint64_t* t,
                              const double* S, const double* S_next, const int32_t* a,
                              const double* r, const uint8_t* term, double* Q_out, double* Qn_out,
                              double* y_out, double* delta_out, double* loss_out,
                              double* grads_out) {
    const uint32_t D = cfg->state_dim, H = cfg->hidden, G = width2(cfg), A = cfg->num_actions;
    const uint32_t B = cfg->batch, O = out_width(cfg);
    const size_t P = oracle_param_count2(D, H, G, O);
    double* eff = effective_params(cfg, params);
    net_view w = view_params(eff, D, H, G, O);

    double* h1 = (double*)malloc((size_t)B * H * sizeof(double));
    double* h2 = (double*)malloc((size_t)B * G * sizeof(double));
    double* Q  = (double*)malloc((size_t)B * A * sizeof(double));
    double* Qn = (double*)malloc((size_t)B * A * sizeof(double));
    forward_with(cfg, eff, S, B, h1, h2, Q);
    if (target_params) {
        double* eff_t = effective_params(cfg, target_params);
        forward_with(cfg, eff_t, S_next, B, NULL, NULL, Qn);
        free(eff_t);
    } else {
        forward_with(cfg, eff, S_next, B, NULL, NULL, Qn);
    }

    /* targets, TD errors, loss, and dL/dQ (one non-zero per row) */
    double* dQ = (double*)calloc((size_t)B * A, sizeof(double));
    double L = 0.0;
    for (uint32_t i = 0; i < B; ++i) {
        double best = Qn[(size_t)i * A];
        for (uint32_t k = 1; k < A; ++k)
            if (Qn[(size_t)i * A + k] > best) best = Qn[(size_t)i * A + k];
        double y = r[i] + cfg->gamma * (term[i] ? 0.0 : 1.0) * best;
        double q = Q[(size_t)i * A + (uint32_t)a[i]];
        double d = y - q;
        L += sample_loss(cfg->loss, d);
        dQ[(size_t)i * A + (uint32_t)a[i]] = -sample_loss_slope(cfg->loss, d) / B;
        if (y_out) y_out[i] = y;
        if (delta_out) delta_out[i] = d;
    }
    L /= B;

    /* gradient at the last layer's outputs: dQ itself, or dQ pulled back through the dueling
     * combine: dV = sum_a dQ[a], dA[a] = dQ[a] - mean_a' dQ[a'] */
    double* dz3 = (double*)calloc((size_t)B * O, sizeof(double));
    for (uint32_t i = 0; i < B; ++i) {
        if (!cfg->dueling) {
            for (uint32_t a = 0; a < A; ++a) dz3[(size_t)i * O + a] = dQ[(size_t)i * A + a];
            continue;
        }
        double sum = 0.0;
        for (uint32_t a = 0; a < A; ++a) sum += dQ[(size_t)i * A + a];
        dz3[(size_t)i * O] = sum;
        for (uint32_t a = 0; a < A; ++a) dz3[(size_t)i * O + 1 + a] = dQ[(size_t)i * A + a] - sum / A;
    }

    double* g = (double*)calloc(P, sizeof(double));
    double* gW1 = g;
    double* gb1 = gW1 + (size_t)D * H;
    double* gW2 = gb1 + H;
    double* gb2 = gW2 + (size_t)H * G;
    double* gW3 = gb2 + G;
    double* gb3 = gW3 + (size_t)G * O;

    /* output layer: dW3 = h2^T dz3 where the head has a weight, db3 = column sums of dz3 */
#pragma omp parallel for schedule(static)
    for (int64_t k = 0; k < (int64_t)G; ++k)
        for (uint32_t i = 0; i < B; ++i)
            for (uint32_t o = 0; o < O; ++o)
                if (head_connected(cfg, (uint32_t)k, o))
                    gW3[(size_t)k * O + o] += h2[(size_t)i * G + k] * dz3[(size_t)i * O + o];
    for (uint32_t i = 0; i < B; ++i)
        for (uint32_t o = 0; o < O; ++o) gb3[o] += dz3[(size_t)i * O + o];

    /* dz2 = (dz3 W3^T) masked by the second ReLU */
    double* dz2 = (double*)malloc((size_t)B * G * sizeof(double));
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < (int64_t)B; ++i)
        for (uint32_t k = 0; k < G; ++k) {
            double acc = 0.0;
            for (uint32_t o = 0; o < O; ++o) acc += dz3[(size_t)i * O + o] * w.W3[(size_t)k * O + o];
            if (!(h2[(size_t)i * G + k] > 0.0)) acc = 0.0;
            dz2[(size_t)i * G + k] = cfg->bf16 ? oracle_round_bf16(acc) : acc;
        }

    /* dW2 = h1^T dz2, db2 = column sums of dz2 */
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < (int64_t)H; ++j)
        for (uint32_t i = 0; i < B; ++i)
            for (uint32_t k = 0; k < G; ++k)
                gW2[(size_t)j * G + k] += h1[(size_t)i * H + j] * dz2[(size_t)i * G + k];
    for (uint32_t i = 0; i < B; ++i)
        for (uint32_t k = 0; k < G; ++k) gb2[k] += dz2[(size_t)i * G + k];

    /* dz1 = (dz2 W2^T) masked by the first ReLU */
    double* dz1 = (double*)malloc((size_t)B * H * sizeof(double));
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < (int64_t)B; ++i)
        for (uint32_t j = 0; j < H; ++j) {
            double acc = 0.0;
            for (uint32_t k = 0; k < G; ++k) acc += dz2[(size_t)i * G + k] * w.W2[(size_t)j * G + k];
            if (!(h1[(size_t)i * H + j] > 0.0)) acc = 0.0;
            dz1[(size_t)i * H + j] = cfg->bf16 ? oracle_round_bf16(acc) : acc;
        }

    /* dW1 = S^T dz1, db1 = column sums of dz1 */
#pragma omp parallel for schedule(static)
    for (int64_t d = 0; d < (int64_t)D; ++d)
        for (uint32_t i = 0; i < B; ++i)
            for (uint32_t j = 0; j < H; ++j)
                gW1[(size_t)d * H + j] += S[(size_t)i * D + d] * dz1[(size_t)i * H + j];
    for (uint32_t i = 0; i < B; ++i)
        for (uint32_t j = 0; j < H; ++j) gb1[j] += dz1[(size_t)i * H + j];

    /* parameter update on the (unrounded) master parameters */
    oracle_opt_apply(cfg, P, params, m, v, t, g);

    if (Q_out) memcpy(Q_out, Q, (size_t)B * A * sizeof(double));
    if (Qn_out) memcpy(Qn_out, Qn, (size_t)B * A * sizeof(double));
    if (loss_out) *loss_out = L;
    if (grads_out) memcpy(grads_out, g, P * sizeof(double));
    free(eff); free(h1); free(h2); free(Q); free(Qn); free(dQ); free(dz3); free(g); free(dz2); free(dz1);
}

void oracle_train_step(const oracle_train_cfg* cfg, double* params, double* m, double* v,
                       uint64_t* t, const double* S, const double* S_next, const int32_t* a,
                       const double* r, const uint8_t* term, double* Q_out, double* Qn_out,
                       double* y_out, double* delta_out, double* loss_out, double* grads_out) {
    oracle_train_step_target(cfg, params, NULL, m, v, t, S, S_next, a, r, term, Q_out, Qn_out, y_out,
                             delta_out, loss_out, grads_out);
}
