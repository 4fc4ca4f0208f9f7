/*
 * CPU oracle for the device-resident experience-replay train step.
 *
 * TEST INFRASTRUCTURE ONLY.  This is a plain, slow, scalar implementation of
 * what the replay (FIFO ring, uniform sampling with replacement, row gather
 * and unpack) and the Q-learning step compute, written straight from the
 * paper (Related Work: experience tuple, FIFO, burn-in; Methods: packed rows,
 * add/sample API, uniform integer sampling; Integration: Q(s,a) selection;
 * Deep Q-Network Model: the update equation; Discussion: one state per
 * experience).  Only tests, the smoke check and the benchmark's cpu_baseline
 * leg may call it.  It shares no code, header, table or constant generator
 * with the GPU library and is never a fallback for it.
 *
 * All floating-point arithmetic of the train step is carried out in double.
 * Exact parts (ring, indices, gathered bytes) are integer / byte work.
 */
#ifndef REPLAY_ORACLE_H
#define REPLAY_ORACLE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* state element types held by a ring */
enum { ORACLE_F32 = 0, ORACLE_BF16 = 1, ORACLE_U8 = 2 };
/* PAIR: every experience stores both states (Methods, packed row of 2D+3).
 * CHAIN: one state per experience, the new state is the next experience's
 * old state (Discussion, halving the memory). */
enum { ORACLE_PAIR = 0, ORACLE_CHAIN = 1 };
enum { ORACLE_HUBER = 0, ORACLE_MSE = 1 };
enum { ORACLE_SGD = 0, ORACLE_ADAM = 1 };

typedef struct oracle_ring oracle_ring;

void oracle_set_threads(int n);
int  oracle_get_threads(void);

/* Philox4x32-10, Salmon et al., SC'11. */
void oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]);

/* The i-th uniform draw from [0, n_choices) of sampling step `step`. */
uint32_t oracle_uniform_index(uint64_t seed, uint64_t step, uint32_t i, uint64_t n_choices);
/* The i-th member (i < n_choices) of a sample of distinct integers from [0, n_choices). */
uint32_t oracle_distinct_index(uint64_t seed, uint64_t step, uint32_t i, uint64_t n_choices);
/* `nsteps` consecutive steps, `batch` draws each: out[k*batch + i]. */
void oracle_uniform_indices(uint64_t seed, uint64_t step0, uint64_t nsteps, uint32_t batch,
                            uint64_t n_choices, uint32_t* out);

oracle_ring* oracle_ring_create(uint64_t capacity, uint32_t state_dim, uint32_t state_dtype,
                                uint32_t layout, uint64_t burn_in);
void oracle_ring_destroy(oracle_ring* ring);
/* n experiences, appended one after the other.  s_next is ignored for CHAIN.
 * Returns 0, or -1 for bad arguments (n > capacity, null pointers). */
int  oracle_ring_append(oracle_ring* ring, uint64_t n, const void* s, const void* s_next,
                        const int32_t* a, const float* r, const uint8_t* term);
void oracle_ring_state(const oracle_ring* ring, uint64_t* head, uint64_t* size, uint64_t* total);
/* Copy n slots starting at first_slot (wrapping) out of the ring, field by field. */
int  oracle_ring_read(const oracle_ring* ring, uint64_t first_slot, uint64_t n, void* s,
                      void* s_next, int32_t* a, float* r, uint8_t* term);
/* Physical slot numbers of one sample.  Returns 0, 1 when sampling is refused
 * (burn-in not complete, or nothing to sample), -1 for bad arguments. */
int  oracle_ring_sample(const oracle_ring* ring, uint64_t seed, uint64_t step, uint32_t batch,
                        uint32_t* idx);
/* The same with distinct != 0: a sample without duplicates (refused, 1, while fewer than
 * `batch` experiences can be drawn). */
int  oracle_ring_sample_mode(const oracle_ring* ring, uint64_t seed, uint64_t step, uint32_t batch,
                             int distinct, uint32_t* idx);
/* Unpack the experiences at idx[] into contiguous batch arrays.  F32 and BF16
 * states are copied bit for bit; U8 states come out as float = u8 / 255. */
int  oracle_ring_gather(const oracle_ring* ring, const uint32_t* idx, uint32_t batch, void* out_s,
                        void* out_s_next, int32_t* out_a, float* out_r, uint8_t* out_term);

/* round-to-nearest-even to bfloat16, returned as the double it represents */
double   oracle_round_bf16(double x);
uint16_t oracle_bf16_bits(float x);

typedef struct {
    uint32_t state_dim, hidden, num_actions, batch;
    uint32_t loss;     /* ORACLE_HUBER | ORACLE_MSE */
    uint32_t opt;      /* ORACLE_SGD | ORACLE_ADAM  */
    uint32_t bf16;     /* 1: apply the bf16 rounding points of the mixed-precision path */
    uint32_t dueling;  /* 1: dueling head (Deep Q-Network Model): Q = V + A - mean A; the last layer
                          has 1 + num_actions outputs (V first), fed by the two halves of the second
                          hidden layer */
    double lr, gamma, beta1, beta2, eps;
    uint32_t hidden2;  /* width of the second hidden layer; 0 = the same as `hidden`.  With the
                          dueling head its two halves are the value and the advantage stream
                          (Deep Q-Network Model: shared layer 128, two streams of 512) */
    uint32_t pad_;
} oracle_train_cfg;

/* Parameters are one flat array: W1[D*H] b1[H] W2[H*G] b2[G] W3[G*A] b3[A] (G = the second
 * hidden width), every matrix row-major [in x out]; with the dueling head W3 and b3 have
 * 1 + num_actions columns, i.e. the count is oracle_param_count2(D, H, G, num_actions + 1). */
size_t oracle_param_count(uint32_t D, uint32_t H, uint32_t A);   /* G = H */
size_t oracle_param_count2(uint32_t D, uint32_t H, uint32_t G, uint32_t A);

/* Q = MLP(X) for n rows of X[n x D]; h1 [n x H], h2 [n x G] (post-ReLU) may be NULL. */
void oracle_mlp_forward(const oracle_train_cfg* cfg, const double* params, const double* X,
                        uint32_t n, double* h1, double* h2, double* Q);

/* mean loss over the batch of (y_i - Q(s_i)[a_i]) with targets y held fixed */
double oracle_loss_fixed_targets(const oracle_train_cfg* cfg, const double* params,
                                 const double* S, const int32_t* a, const double* y);

/* The parameter update alone, from a given gradient of the mean loss: SGD, or Adam with bias
 * correction (t is advanced first).  params, m, v [n] are updated in place. */
void oracle_opt_apply(const oracle_train_cfg* cfg, size_t n, double* params, double* m, double* v,
                      uint64_t* t, const double* g);

/* One Q-learning step on a batch.  params (and m, v, t for Adam) are updated in
 * place.  Optional outputs (NULL to skip): Q[B*A], Qn[B*A], y[B], delta[B],
 * loss[1], grads[param_count]. */
void oracle_train_step(const oracle_train_cfg* cfg, double* params, double* m, double* v,
                       uint64_t* t, const double* S, const double* S_next, const int32_t* a,
                       const double* r, const uint8_t* term, double* Q, double* Qn, double* y,
                       double* delta, double* loss, double* grads);

/* The same with a frozen target network for Q(s', .) (NULL = the trained network). */
void oracle_train_step_target(const oracle_train_cfg* cfg, double* params,
                              const double* target_params, double* m, double* v, uint64_t* t,
                              const double* S, const double* S_next, const int32_t* a,
                              const double* r, const uint8_t* term, double* Q, double* Qn,
                              double* y, double* delta, double* loss, double* grads);

#ifdef __cplusplus
}
#endif
#endif
