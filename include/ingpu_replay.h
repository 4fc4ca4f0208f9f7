/*
 * ingpu_replay — device-resident experience replay and Q-learning train step
 * for AMD MI355X (gfx950).  Plain C ABI.
 *
 * The interface follows the paper's problem statement: an experience replay
 * with two methods, "add" and "sample" (Methods), whose sample call returns
 * old state, new state, action, reward and is_terminal tensors with all type
 * casting hidden from the user (Methods), and a train step that takes no
 * network inputs from the host (Integration with Reinforcement Learning
 * Algorithm).
 *
 * Conventions
 *  - Ownership: the caller allocates every device buffer (ring storage,
 *    trainer workspace, sample outputs) and keeps it alive until the matching
 *    *_destroy call.  The library owns only its host-side handles, pinned host
 *    buffers for host-sourced experiences (a few times max_append rows per replay,
 *    a few dozen steps' worth per trainer), and its HIP graph objects.
 *  - Streams: `hip_stream` is a hipStream_t passed as void* (NULL = the null
 *    stream).  All calls are asynchronous on that stream except the ones marked
 *    "synchronises", which exist for tests and inspection.  One handle must be
 *    driven from one stream at a time.
 *  - Status: 0 = done, > 0 = benign (nothing was sampled or trained),
 *    < 0 = failure; a failing call changes no replay or trainer state.  A
 *    message for the last failure on the calling thread is returned by
 *    rp_last_error().  Nothing throws across this boundary.
 *  - "device" / "host" below say where a pointer must point.
 */
#ifndef INGPU_REPLAY_H
#define INGPU_REPLAY_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct replay  replay_t;  /* opaque host handle */
typedef struct trainer trainer_t; /* opaque host handle */

typedef enum {
    RP_OK = 0,
    RP_SKIPPED_BURN_IN = 1, /* burn-in not complete (Related Work: no training during burn-in),
                               or nothing to sample yet */
    RP_EINVAL = -1,         /* null pointer, zero size, size beyond a limit, mismatched dims */
    RP_ENOMEM = -2,         /* a caller-provided buffer is too small / host allocation failed */
    RP_EHIP = -3,           /* a HIP runtime call failed; see rp_last_error() */
    RP_ESTATE = -4          /* device-resident state disagrees with the host mirror */
} rp_status;

/* element type of a stored state */
enum { RP_F32 = 0, RP_BF16 = 1, RP_U8 = 2 };
/* RP_PAIR: an experience stores both states, one packed row
 *          [s(D) | s'(D) | action | reward | is_terminal] (Methods: rows of 2D+3 values).
 * RP_CHAIN: one state per experience; the new state of slot p is the state in
 *          slot p+1 (Discussion: halves the memory when states are large). */
enum { RP_PAIR = 0, RP_CHAIN = 1 };
enum { RP_HUBER = 0, RP_MSE = 1 };
enum { RP_SGD = 0, RP_ADAM = 1 };
/* train_config.flags: GRAPH = an executed step is replayed as one HIP graph launch;
 * LAYERED = always use the one-kernel-per-layer step, also where the two-kernel step for
 * small fp32 networks would apply (both give the same results to rounding). */
enum { RP_TRAIN_GRAPH = 1, RP_TRAIN_LAYERED = 2 };
/* replay_config.sampling.  RP_WITH_REPLACEMENT: every draw independent (Methods: what the
 * in-GPU replay does; a batch may repeat an experience).  RP_DISTINCT: a batch never repeats an
 * experience (Methods: what the in-RAM replay does and the author wants back). */
enum { RP_WITH_REPLACEMENT = 0, RP_DISTINCT = 1 };
/* train_config.head.  RP_HEAD_PLAIN: the last layer gives Q(s, .) directly.  RP_HEAD_DUELING: the
 * dueling head of the paper's network (Deep Q-Network Model): the second hidden layer is two
 * streams side by side, units 0 .. G/2-1 feed a state value V, units G/2 .. G-1 feed one
 * advantage per action (G = the second hidden layer's width), and
 * Q(s,a) = V(s) + A(s,a) - mean_a' A(s,a').  The last layer then has 1 + num_actions outputs
 * (V first) in every parameter array: W3[G*(1+A)] b3[1+A]; its weights from the other stream's
 * units take no part and never change. */
enum { RP_HEAD_PLAIN = 0, RP_HEAD_DUELING = 1 };

typedef struct {
    uint64_t capacity;    /* number of experiences the replay holds (1,000,000 in the paper) */
    uint32_t state_dim;   /* D: elements per state (27 in the paper)                          */
    uint32_t state_dtype; /* RP_F32 | RP_BF16 | RP_U8                                         */
    uint32_t layout;      /* RP_PAIR | RP_CHAIN                                               */
    uint32_t max_append;  /* largest n a host-sourced replay_append moves in one piece; the
                             storage holds a device staging area of this many rows (>= 1)     */
    uint64_t burn_in;     /* sampling and training are refused until this many experiences
                             have been added in total                                         */
    uint64_t seed;        /* key of the index generator                                       */
    uint32_t sampling;    /* RP_WITH_REPLACEMENT | RP_DISTINCT                                */
    uint32_t reserved;    /* 0                                                                */
} replay_config;

/* Bytes of device memory replay_create needs for this configuration (0 if the
 * configuration is invalid).  Pure host arithmetic.  (Methods: the replay is one device-resident
 * array of capacity x (2D+3) values, 1,000,000 x 57 floats in the paper; here each row is padded,
 * see replay_row_bytes, and a small state block and staging area precede the rows.) */
size_t replay_storage_bytes(const replay_config* cfg);

/* Bytes of one stored experience.  PAIR (Methods: a row packs both states, action, reward and
 * is_terminal, 2D+3 values): the packed row padded to 16, 32 or 64 bytes or to a multiple of
 * 128 bytes, 256 for the paper's 57 floats.  CHAIN (Discussion: one state per experience): the
 * state padded the same way plus 9 bytes of side data (action, reward, is_terminal).
 * Pure host arithmetic; 0 if invalid. */
size_t replay_row_bytes(const replay_config* cfg);

/*
 * Create an empty replay (Methods: fixed size, starts empty) inside
 * `dev_storage` (device, 256-byte aligned, at least replay_storage_bytes()).
 * The storage is cleared.  Synchronises.
 */
rp_status replay_create(const replay_config* cfg, void* dev_storage, size_t bytes,
                        replay_t** out);

/* Release the host handle.  Never frees dev_storage. */
rp_status replay_destroy(replay_t* rp);

/*
 * "Add" (Methods): append n experiences in first-in first-out order,
 * overwriting the oldest once the replay is full; a batch that reaches the end
 * of the storage wraps to slot 0.  Arrays are structure-of-arrays, row-major:
 * s[n*D], s_next[n*D] of the state type (s_next is ignored and may be NULL for
 * RP_CHAIN), a[n], r[n], term[n] (any non-zero byte = terminal).
 * src_is_device = 0: host pointers, copied into pinned memory in pieces of
 * max_append rows, from where the append kernel reads them (the arrays may be
 * reused as soon as the call returns); 1: device pointers, read directly by the append kernel and
 * to be left untouched until the stream reaches it.  n = 0 is a no-op; n >
 * capacity is RP_EINVAL.
 */
rp_status replay_append(replay_t* rp, uint64_t n, const void* s, const void* s_next,
                        const int32_t* a, const float* r, const uint8_t* term, int src_is_device,
                        void* hip_stream);

/*
 * "Sample" (Methods): draw `batch` slot numbers uniformly, with replacement,
 * from the experiences currently held, and unpack those experiences into
 * contiguous batch tensors (all device pointers):
 *   out_s[batch*D], out_s_next[batch*D]  float for RP_F32 states, bf16 bits for
 *                                        RP_BF16, float = u8/255 for RP_U8;
 *   out_a[batch] int32, out_r[batch] float, out_term[batch] 0/1 bytes;
 *   out_idx[batch] the sampled slot numbers (may be NULL).
 * Draw i of a call is a pure function of (seed, step, i, current size): word
 * i mod 4 of Philox4x32-10 with key = seed and counter = (i div 4, 0, step),
 * mapped to floor(word * size / 2^32).  RP_CHAIN draws among the size-1
 * experiences that already have a successor.  For RP_CHAIN, out_s_next of a
 * terminal experience holds the next slot's state and is to be masked by the
 * caller with out_term.
 * With RP_DISTINCT, draw i is instead the image of i under a keyed permutation of the
 * choices: a swap-or-not shuffle of 2*bitlen(choices-1)+8 rounds driven by the same
 * generator (round r: partner K_r - x mod choices with K_r from word r mod 4 of counter
 * (r div 4, 1, step); swap bit = bit 0 of word 0 of counter (max(x, partner), 2 + r, step)).
 * Returns RP_SKIPPED_BURN_IN, writing nothing, before burn-in completes, while there is
 * nothing to sample, or (RP_DISTINCT) while fewer than `batch` experiences can be drawn.
 * batch = 0 or batch > 2^24 is RP_EINVAL.
 */
rp_status replay_sample_gather(replay_t* rp, uint64_t step, uint32_t batch, void* out_s,
                               void* out_s_next, int32_t* out_a, float* out_r, uint8_t* out_term,
                               uint32_t* out_idx, void* hip_stream);

/*
 * replay_sample_gather for callers that cannot allocate device memory or accept a library that
 * does: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments, same results.  The one scratch buffer the call needs (the slot numbers of a
 * batch without duplicates, handed from the kernel that draws them to the kernel that gathers)
 * is a fixed 256 KB array inside the library's own image instead of part of dev_storage, so the
 * call allocates nothing and calls no allocating routine.  Limits and rules:
 *  - RP_DISTINCT replays: batch <= 65,536 (the array's size), else RP_EINVAL; RP_WITH_REPLACEMENT
 *    replays need no scratch and have no extra limit.
 *  - every GPU the library runs on holds its own copy of the array until the process ends;
 *    all calls on one GPU share it.  Nothing in it has to be cleared between calls (a call
 *    writes every word it later reads), but two calls that overlap in time on the same GPU, from
 *    different streams or handles, race on it: serialise them (one stream, or events).
 */
rp_status replay_sample_gather_static(replay_t* rp, uint64_t step, uint32_t batch, void* out_s,
                                      void* out_s_next, int32_t* out_a, float* out_r,
                                      uint8_t* out_term, uint32_t* out_idx, void* hip_stream);

/* Write position, number of experiences held, and experiences ever added, as
 * read back from the device.  RP_ESTATE if they differ from the host mirror.
 * Synchronises the device. */
rp_status replay_get_state(replay_t* rp, uint64_t* head, uint64_t* size, uint64_t* total);

/* Copy n stored experiences starting at slot first_slot (wrapping) to host
 * arrays, field by field (any may be NULL; s_next is not written for
 * RP_CHAIN).  States come back in their stored type.  Synchronises. */
rp_status replay_read_rows(replay_t* rp, uint64_t first_slot, uint64_t n, void* s, void* s_next,
                           int32_t* a, float* r, uint8_t* term);

typedef struct {
    uint32_t state_dim;        /* D, must equal the replay's                                   */
    uint32_t hidden;           /* H: width of the two hidden layers (multiple of 64)           */
    uint32_t num_actions;      /* A                                                            */
    uint32_t batch;            /* B experiences per train step                                 */
    uint32_t param_dtype;      /* RP_F32: fp32 everywhere (replay states RP_F32);
                                  RP_BF16: bf16 matrix inputs with fp32 accumulation and fp32
                                  master weights (replay states RP_BF16)                       */
    uint32_t loss;             /* RP_HUBER (threshold 1) | RP_MSE (half squared error)         */
    uint32_t opt;              /* RP_SGD | RP_ADAM                                             */
    uint32_t appends_per_step; /* experiences added by every train_step (0 = none)             */
    float lr, gamma, beta1, beta2, eps;
    uint32_t flags;            /* RP_TRAIN_GRAPH | RP_TRAIN_LAYERED                            */
    uint32_t target_sync;      /* 0: Q(s',.) comes from the trained network itself (the update
                                  equation as printed).  N > 0: from a frozen copy of the weights
                                  that is overwritten with the trained ones after every N-th
                                  update (Deep Q-Network Model: target fixing, N = 10,000)      */
    uint32_t head;             /* RP_HEAD_PLAIN | RP_HEAD_DUELING                              */
    uint32_t hidden2;          /* G: width of the second hidden layer (multiple of 64); 0 = H.
                                  The paper's network (Deep Q-Network Model: a shared layer of 128
                                  units, then a value and an advantage stream of 512 units each)
                                  is hidden = 128, hidden2 = 1024, head = RP_HEAD_DUELING          */
} train_config;

/* number of network parameters: D*H + H + H*G + G + G*O + O, O = A (plain head) or 1 + A (dueling) */
size_t train_param_count(const train_config* cfg);
/* Bytes of device workspace train_create needs (0 if the configuration is invalid). */
size_t train_workspace_bytes(const train_config* cfg);

/*
 * Create a trainer for the network D -> H -> G -> A (ReLU after both hidden
 * layers; G = hidden2, or H when that is 0) on top of a PAIR replay.  host_init_params (host)
 * holds W1[D*H] b1[H] W2[H*G] b2[G] W3[G*A] b3[A], matrices row-major [in x out].
 * dev_workspace: device, 256-byte aligned, train_workspace_bytes().  Synchronises.
 */
rp_status train_create(const train_config* cfg, replay_t* rp, void* dev_workspace, size_t bytes,
                       const float* host_init_params, trainer_t** out);
rp_status train_destroy(trainer_t* tr);

/*
 * With target_sync = N > 0 the target network starts as a copy of host_init_params; it is synced
 * when the number of updates applied so far (Adam's t, counted for SGD too) is a multiple of N.
 *
 * One train step with no network inputs from the host (Integration): append
 * appends_per_step experiences (arrays as in replay_append; ignored when
 * appends_per_step = 0), then, once burn-in is complete, sample a batch with
 * the trainer's own step counter (starts at 0, advances on executed steps
 * only), gather it, run the network on s and s', form
 *   y = r + gamma (1 - terminal) max_a' Q(s',a'),  delta = y - Q(s,a)
 * (Deep Q-Network Model, the update equation, with the target held constant),
 * take the mean Huber / half-squared loss, backpropagate through Q(s,.) and
 * apply SGD or Adam.  Returns RP_SKIPPED_BURN_IN when only the append ran.
 */
rp_status train_step(trainer_t* tr, const void* s, const void* s_next, const int32_t* a,
                     const float* r, const uint8_t* term, int src_is_device, void* hip_stream);

/*
 * `count` consecutive train steps in one call: step k consumes experiences
 * k*appends_per_step .. (k+1)*appends_per_step - 1 of the given arrays (which hold
 * count*appends_per_step experiences).  Same semantics as calling train_step `count`
 * times; *executed (may be NULL) receives the number of steps that trained.
 */
rp_status train_steps(trainer_t* tr, uint64_t count, const void* s, const void* s_next,
                      const int32_t* a, const float* r, const uint8_t* term, int src_is_device,
                      void* hip_stream, uint64_t* executed);

/*
 * One train step on a batch the caller provides instead of a sampled one: device arrays of
 * `batch` experiences, structure of arrays as replay_sample_gather writes them (states in the
 * replay's state type).  Nothing is appended or drawn; the rest of the step is the one of
 * train_step (Deep Q-Network Model, the update equation), the trainer's step counter advances,
 * and train_get_last reports 0..batch-1 as the slot numbers.  This is the step the in-RAM
 * comparison system below feeds.
 */
rp_status train_step_batch(trainer_t* tr, const void* s, const void* s_next, const int32_t* a,
                           const float* r, const uint8_t* term, void* hip_stream);

/* Test / inspection calls; host destinations, any may be NULL; all synchronise.
 * train_get_opt_state and train_get_last return RP_ESTATE (outputs filled all the same) if a
 * train step with a target network has run whose workgroups did not receive the target
 * network's values from their partner workgroups within the kernel's time limit (the step then
 * used zeros): the trainer's weights are not to be trusted from that step on. */
rp_status train_get_params(trainer_t* tr, float* params);             /* fp32 master weights */
rp_status train_get_grads(trainer_t* tr, float* grads);               /* of the last step    */
rp_status train_get_opt_state(trainer_t* tr, float* m, float* v, uint64_t* t, uint64_t* step);
/* The frozen target network's weights (same order as train_get_params); equal to the trained
 * weights when target_sync = 0.  train_set_target is RP_EINVAL when target_sync = 0. */
rp_status train_get_target(trainer_t* tr, float* params);
rp_status train_set_target(trainer_t* tr, const float* params);
/* Overwrite weights, Adam moments (NULL = keep), Adam t and the sampling step counter.  The
 * target network is left as it is. */
rp_status train_set_state(trainer_t* tr, const float* params, const float* m, const float* v,
                          uint64_t t, uint64_t step);
/* From the last executed step: Q(s,.) [B*A], Q(s',.) [B*A], y[B], delta[B], loss[1],
 * sampled slot numbers idx[B]. */
rp_status train_get_last(trainer_t* tr, float* q, float* q_next, float* y, float* delta,
                         float* loss, uint32_t* idx);
/* Test call for the bounded wait above.  ticks: the longest a workgroup waits for its partner, in
 * ticks of the GPU's 100 MHz wall clock (0 = the default, 50 ms; at most 2^40).  break_pairing
 * != 0 makes the waiting workgroups of later steps look for a launch number that no workgroup
 * sends, so every wait runs out after `ticks`: the kernels end normally, the steps compute with
 * zeros in place of the target network's values, and the read-back calls return RP_ESTATE until
 * train_set_state (which clears the mark) is called.  Takes effect from the next step enqueued. */
rp_status train_set_handoff_wait(trainer_t* tr, uint64_t ticks, int break_pairing);
/* Test call.  Two-kernel step with a target network: whether the last executed step took
 * max_a Q_target(s', a) of its experience 0 from the table that the step before it filled
 * (*from_table = 1) or had it computed inside its own launch (0).  Synchronises. */
rp_status train_get_target_source(trainer_t* tr, uint32_t* from_table);
/* Number of GPU kernels one executed train step launches (graph nodes). */
rp_status train_kernels_per_step(trainer_t* tr, uint32_t* n);

/*
 * The paper's comparison system, re-created for measurement: an experience replay kept in host
 * RAM (Methods and Results: the "in-RAM" replay).  float32 states, both states stored.  Each
 * train step draws its batch on the host with the same generator, key and counter layout as
 * replay_sample_gather (so it trains on the same batches as the device-resident replay),
 * gathers the rows into pinned memory, copies the batch to the GPU and calls train_step_batch.
 * dev_batch: device memory of inram_device_bytes(state_dim, batch) bytes, 256-byte aligned,
 * owned by the caller.  The trainer passed to the step calls must have been created with the
 * same state_dim and batch.
 */
typedef struct inram_replay inram_replay_t;
size_t    inram_device_bytes(uint32_t state_dim, uint32_t batch);
rp_status inram_create(uint64_t capacity, uint32_t state_dim, uint64_t burn_in, uint64_t seed,
                       uint32_t batch, void* dev_batch, size_t bytes, inram_replay_t** out);
rp_status inram_destroy(inram_replay_t* h);
/* host arrays, structure of arrays; FIFO with wraparound as replay_append */
rp_status inram_append(inram_replay_t* h, uint64_t n, const float* s, const float* s_next,
                       const int32_t* a, const float* r, const uint8_t* term);
/* RP_SKIPPED_BURN_IN (nothing done) before burn-in completes; sampling step counter starts at 0 */
rp_status inram_train_step(inram_replay_t* h, trainer_t* tr, void* hip_stream);
/* count x (append appends_per_step experiences from the host arrays, then one train step) */
rp_status inram_train_steps(inram_replay_t* h, trainer_t* tr, uint64_t count,
                            uint32_t appends_per_step, const float* s, const float* s_next,
                            const int32_t* a, const float* r, const uint8_t* term, void* hip_stream,
                            uint64_t* executed);
rp_status inram_get_state(inram_replay_t* h, uint64_t* head, uint64_t* size, uint64_t* total,
                          uint64_t* step);

/* Message for the last failure on this thread ("" if none). */
const char* rp_last_error(void);
/* Library version string. */
const char* rp_version(void);

#ifdef __cplusplus
}
#endif
#endif /* INGPU_REPLAY_H */
