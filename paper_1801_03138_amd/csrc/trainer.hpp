// Shared definitions of the trainer: element types, device-resident counters, the host handle.
#pragma once

#include <cmath>

#include "common.hpp"

namespace rp {

constexpr unsigned int kTrainThreads = 256;

// ----------------------------------------------------------------------------- element types
struct bf16_t {
    unsigned short bits;
};

__device__ __forceinline__ float to_float(float x) { return x; }
__device__ __forceinline__ float to_float(bf16_t x) {
    return __uint_as_float((unsigned int)x.bits << 16);
}
// round to nearest even; NaN stays NaN
__device__ __forceinline__ unsigned short bf16_bits_rne(float f) {
    unsigned int u = __float_as_uint(f);
    if ((u & 0x7F800000u) == 0x7F800000u && (u & 0x007FFFFFu)) return (unsigned short)((u >> 16) | 0x40u);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (unsigned short)(u >> 16);
}
template <typename T>
__device__ __forceinline__ T from_float(float x);
template <>
__device__ __forceinline__ float from_float<float>(float x) { return x; }
template <>
__device__ __forceinline__ bf16_t from_float<bf16_t>(float x) { return bf16_t{bf16_bits_rne(x)}; }

// Device-resident scalars of the trainer.
struct TrainCounters {
    unsigned long long step;    // sampling step of the next executed train step
    unsigned long long adam_t;  // Adam steps taken
    float c1, c2;               // Adam bias corrections 1 - beta^t of the current step
    float loss;                 // mean loss of the last step
    unsigned int handoff_missed;   // set when a workgroup's bounded wait for another one ran out
    double pw1, pw2;            // beta1^t, beta2^t for t = adam_t (kept by the steps that advance t on the device)
    unsigned int from_table;    // last step, experience 0: target value taken from the table filled a step ahead
    unsigned int pad_[3];
};
static_assert(sizeof(TrainCounters) == 64, "one line");


// Whether the dueling head has a weight from unit k of the second hidden layer (H units; k = H:
// the bias) to output o (0 = state value, fed by units 0 .. H/2-1; 1 + a = advantage of action a,
// fed by the rest).
__host__ __device__ inline bool head_connected(unsigned int H, unsigned int k, unsigned int o) {
    if (k >= H) return true;
    return o == 0 ? k < H / 2 : k >= H / 2;
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
    return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}


// Argument block of the fused row kernel.
struct RowArgs {
    RingGeom g;
    unsigned long long seed;
    unsigned int n_append;
    unsigned int append_group;   // the launch has a workgroup for the append (trainers that append at all)
    Payload src;          // this step's new experiences
    Payload batch;        // from_batch: the batch itself, given by the caller instead of sampled
    unsigned int from_batch;
    // ring and trainer state before this step, from the host mirror (set before every launch,
    // so the kernel can start drawing without a dependent load)
    unsigned long long head, step;
    unsigned int size_after;     // experiences held once this step's append is in
    unsigned long long total_after, adam_t_after;   // experiences ever added / Adam steps, after this step
    float c1_after, c2_after;    // Adam's bias corrections 1 - beta^t for that step count
    // Sampling without duplicates: an extra workgroup draws the NEXT step's slots while this step
    // runs (a draw is a long chain of dependent Philox blocks).  pre holds two buffers of
    // pre_stride words, [step lo, step hi, size, -, slots...], used alternately by step parity; a
    // step takes its slots from there when step and size match and draws them itself otherwise.
    unsigned int* pre;           // null: no extra workgroup, no look-up
    unsigned int pre_stride;
    unsigned int next_size;      // experiences held after the next step's append
    // Target network in workgroups of its own: max_a Q_target(s'_i, a) travels from one workgroup to
    // another inside the launch as handoff[i] = (seq << 32) | float bits; seq differs from launch
    // to launch, so a word left by an earlier launch is never taken for this one's.
    unsigned long long* handoff; // [B]
    unsigned int seq;            // what the sending workgroups stamp their words with
    unsigned int seq_wait;       // what the waiting ones look for (the same, except in a test of the time limit)
    long long handoff_ticks;     // longest wait, in ticks of the 100 MHz wall clock
    // ... and from one launch to the next: table[parity of the step][i] = eight words (the step the
    // entry holds for: sampling step, experiences ever added, Adam steps, each after that step, two
    // words each; count of calls that changed weights from outside; the maximum), with the rows
    // Q_target(s'_i, .) beside it.
    unsigned int* ahead;         // [2][B][8]
    float* qn_ahead;             // [2][B][Ap]
    unsigned int ahead_on;       // fill the table for the next step (the target network stays as it is until then)
    unsigned int epoch;          // calls that changed weights or counters from outside, so far
    unsigned long long next_total_after;   // experiences ever added, after the next step's append
    TrainCounters* ctr;
    const float* w;       // padded parameters
    const float* wt;      // the frozen target network's (Q(s', .) is computed with them), or null
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

// The Adam step count after a step and its bias corrections (the host mirrors the count, so
// the device never evaluates a power).
inline void set_adam_step(RowArgs& a, unsigned long long t_after, float beta1, float beta2) {
    a.adam_t_after = t_after;
    a.c1_after = (float)(1.0 - std::pow((double)beta1, (double)t_after));
    a.c2_after = (float)(1.0 - std::pow((double)beta2, (double)t_after));
}


// Buffers of the mixed-precision step on MFMA (bf16 bit patterns).  "T" = transposed: the
// batch index is the contiguous one, rows are padded to Bp (a multiple of 128) with zeros.
struct WideBuffers {
    unsigned short *W1T, *W2, *W2T, *W3T;   // [H x Dp], [H x H], [H x H] transposed, [Ap x H]
    unsigned short *W1T_t, *W2T_t, *W3T_t;  // forward operands of the frozen target network
    unsigned short* XT;                      // [>= D+1 x Bp], row D all ones
    unsigned short *H1T, *H2T;               // [H+1 x Bp], row H all ones
    unsigned short *dQT_hi, *dQT_lo;         // [Ap x Bp] each, dQT_lo right after dQT_hi
    unsigned short *dZ2T, *dZ1T;             // [H x Bp]
    float* part3;                            // K-split partials [splits][H+1][2 Ap] of [dW3 ; db3]
    float* part1;                            // K-split partials [splits][H][Dx] of [dW1^T | db1]
    float* part2;                            // K-split partials [splits][H+1][H] of [dW2 ; db2]
};

// train_steps runs several steps per graph launch (a launch costs about 5 us of GPU idle time:
// measured 59.8k / 61.5k / 62.0k steps/s with 8 / 16 / 32 steps per launch): graphs of these many
// steps are recorded, longest first, and a run of steps takes the longest that still fits.
// New experiences staged from host memory go 8 at most per launch (16 lost 17 % there).
constexpr unsigned int kRunSteps[] = {32, 16, 8, 4, 2};
constexpr unsigned int kRuns = sizeof(kRunSteps) / sizeof(kRunSteps[0]);
constexpr unsigned int kRunStepsMax = 32, kRunStepsHostPayload = 8;
constexpr unsigned int kPinSlots = 64;       // pinned host slots for host-sourced payloads
constexpr unsigned int kPinGroup = 16;       // slots per completion event

}  // namespace rp

struct trainer {
    train_config cfg;
    replay* rp_;
    unsigned int Dp, Ap, H, B, Bp;   // H: width of the first hidden layer
    unsigned int Hb;                 // width of the second hidden layer (= H unless cfg.hidden2 says otherwise)
    size_t n_params, n_padded;       // external / padded parameter counts
    // Dueling head: the arrays w, g, m, v, wt each continue past their n_padded entries with the
    // head's own parameters [(H+1) x (1+A)] (row H = biases); positions oW3.. / ob3.. of w then
    // hold the equivalent plain output layer W[k][a] = V[k] + A[k][a] - mean_a' A[k][a'], which
    // is all the forward and backward kernels see.
    bool dueling;
    size_t n_head, n_dev;            // head parameters; entries per device array (n_padded + n_head)
    size_t oW1, ob1, oW2, ob2, oW3, ob3;
    size_t elem;                     // bytes of an activation element
    unsigned char* ws;
    rp::TrainCounters* ctr;
    float *w, *g, *m, *v;
    float* wt;                       // frozen target network (padded, as w); null without one
    float* w2t;                      // two-kernel step: W2 transposed, [Hb x H]; fp32 step on MFMA: the copy of W2
                                     // ([H x Hb], made anew in every step) that the dZ1 product reads while
                                     // the second layer's tiles update W2 in place
    rp::bf16_t* wb;
    rp::bf16_t* wbt;                 // layered mixed precision: bf16 copy of the target network
    void* X;                         // [2B x Dp]
    int* act;
    float* rew;
    unsigned char* term;
    unsigned int* idx;
    void *H1, *H2;                   // [2B x H], [2B x Hb]
    float* Q;                        // [2B x Ap]
    float *y, *delta, *lossi, *dQ;   // [B], [B], [B], [B x Ap]
    void *dZ2, *dZ1;                 // [B x Hb], [B x H]
    unsigned int* pre;               // slots drawn ahead, 2 x (4 + B) words
    float* qpart;                    // [8][2B x Ap] partial products of the output layer (fp32 step on MFMA)
    unsigned long long* handoff;     // [B] words one workgroup of the row kernel hands to another
    unsigned int launch_seq;         // number of the last row-kernel launch prepared (never 0)
    long long handoff_ticks;         // longest wait of a workgroup for its partner (wall-clock ticks)
    unsigned int* ahead;             // target values a step ahead, 2 x B x 8 words ...
    float* qn_ahead;                 // ... and 2 x B x Ap
    unsigned int epoch;              // calls that changed weights or counters from outside (never 0)
    bool handoff_break;              // test of that limit: the waiting side expects a number nobody sends
    bool fused;                      // two-kernel step for small fp32 networks
    bool wide;                       // mixed-precision step on MFMA
    bool mid;                        // fp32 step on MFMA, one product per kernel
    rp::WideBuffers wd;
    hipGraph_t graph;
    hipGraphExec_t graph_exec;
    hipStream_t capture_stream;
    unsigned int kernels_per_step;
    uint64_t host_step;              // mirror of ctr->step
    uint64_t host_adam_t;            // mirror of ctr->adam_t
    // The kernel that consumes the step's new experiences (fused row kernel, or the append
    // kernel of the layered step): host copy of its argument block, and its node in the graph,
    // whose argument is replaced before every launch.
    rp::RowArgs row_args;
    rp::AppendGatherArgs append_args;   // the append kernel reads its leading AppendArgs part
    void* payload_func;
    void* payload_kargs[1];          // -> row_args / append_args
    hipGraphNode_t payload_node[1];
    hipKernelNodeParams payload_np[1];
    // Runs of consecutive steps recorded as one graph each, for train_steps: one launch (and one
    // launch gap on the GPU) per run; each step's payload kernel has its own node.
    struct StepRun {
        hipGraph_t graph;
        hipGraphExec_t exec;
        hipGraphNode_t node[rp::kRunStepsMax];
        hipKernelNodeParams np[rp::kRunStepsMax];
    } runs[rp::kRuns];
    // Steps on MFMA with new experiences every step and sampling with replacement: in a recorded
    // run only the first step has an append + gather kernel of its own; the gather of step k + 1
    // is done by extra workgroups of step k's last kernel (the weights kernel of the fp32 step,
    // the optimizer kernel of the mixed-precision step; the run's node k + 1 is that kernel then).
    // The fp32 step's weights kernel still reads the batch, so its steps alternate between two
    // batch buffers (X_buf); the mixed-precision step has one (both entries the same).
    bool gather_ahead;
    void* X_buf[2];
    bool rec_skip_gather;                    // recording: this step's batch was gathered by the step before
    const rp::AppendGatherArgs* rec_next;    // recording: the next step's gather, for this step's weights kernel
    unsigned int rec_parity;                 // recording: which batch buffer this step reads
    void* w_args_host[2];                    // the weights kernel's argument block as recorded, per batch buffer
    // Host-sourced payloads are copied into a ring of pinned, device-mapped host slots that the
    // kernel reads directly; an event per group of slots tells when a group may be reused.
    unsigned char* pin_host;
    unsigned char* pin_dev;
    size_t pin_slot_bytes, pin_off_s_next, pin_off_a, pin_off_r, pin_off_term;
    uint64_t pin_next;
    hipEvent_t pin_event[rp::kPinSlots / rp::kPinGroup];
    bool pin_event_live[rp::kPinSlots / rp::kPinGroup];
};

namespace rp {
// Whether the two-kernel fused step can run this configuration.
bool fused_step_supported(const train_config& cfg, const replay* rp_);
// Dynamic LDS bytes its row kernel needs.
// Enqueue the fused step (append + sample + gather + forward + TD + backward; weight
// gradients + optimizer).  *count receives the number of kernels launched.
// With `batch` the step trains on the caller's batch: nothing is appended or sampled.
hipError_t enqueue_fused_step(trainer* t, const Payload& src, const Payload* batch, hipStream_t st,
                              unsigned int* count);
hipError_t fused_init();                      // once, at trainer creation
// The number that tells one launch of the row kernel from the others (never 0, the value of a
// cleared hand-over word).
// ... and what the target network's workgroups need to know about the step after this one.
// Call with the step's other fields (n_append, from_batch, total_after, adam_t_after) in place.
inline void stamp_launch(trainer* t, RowArgs& a) {
    if (++t->launch_seq == 0) ++t->launch_seq;
    a.seq = t->launch_seq;
    a.seq_wait = t->handoff_break ? ~a.seq : a.seq;
    a.handoff_ticks = t->handoff_ticks;
    a.handoff = t->handoff;
    a.ahead = t->ahead;
    a.qn_ahead = t->qn_ahead;
    a.epoch = t->epoch;
    a.next_total_after = a.total_after + a.n_append;
    // the next step finds the target network as this launch does unless this step's update syncs it
    a.ahead_on = t->wt && !a.from_batch && t->rp_->cfg.sampling == RP_WITH_REPLACEMENT &&
                 a.adam_t_after % t->cfg.target_sync != 0;
}
constexpr long long kHandoffTicks = 5000000;   // default limit: 50 ms
void* fused_rows_func(bool target_network, unsigned int Dp, unsigned int B);   // the row kernel variant for a configuration
// Dueling head: turn the gradient of the equivalent plain output layer (in g) into the head's
// update and refresh that layer (and its bf16 / target copies).  No-op for a plain head.
hipError_t enqueue_head_update(trainer* t, hipStream_t st, unsigned int* count);
// The second kernel of the fused step on its own: weight gradients of all three layers from the
// activations and pre-activation gradients in the workspace, optimizer, mean loss, step counter;
// a dueling head of up to 32 actions is updated by it too (*folded_head says so).
struct MmArgs;
hipError_t enqueue_weights_update(trainer* t, hipStream_t st, bool* folded_head, const MmArgs* dz1 = nullptr,
                                  unsigned int* launches = nullptr);
// The weights kernel with the next step's gather in its launch (see trainer::gather_ahead): its
// __global__ function, replacing the next step's part of a recorded node's arguments, and
// releasing the recorded argument blocks.
void* weights_ahead_func(const trainer* t);
hipError_t patch_weights_ahead_node(trainer* t, hipGraphExec_t exec, hipGraphNode_t node,
                                    const hipKernelNodeParams& recorded, unsigned int parity,
                                    const AppendGatherArgs& next);
void free_weights_args(trainer* t);
// The same for the mixed-precision step, whose last kernel is the optimizer's.
void* opt_ahead_func();
hipError_t patch_opt_ahead_node(trainer* t, hipGraphExec_t exec, hipGraphNode_t node,
                                const hipKernelNodeParams& recorded, const AppendGatherArgs& next);
// fp32 step on MFMA for shapes the two-kernel step does not take (wider layers, two different
// hidden widths): one product per kernel.
bool mid_step_supported(const train_config& cfg, const replay* rp_);
hipError_t enqueue_mid_step(trainer* t, hipStream_t st, unsigned int* count);
unsigned int mid_step_kernels(const trainer* t);   // launches per step, the append + gather kernel included
// Mixed-precision step on MFMA (bf16 replay states and matrix operands).
bool wide_step_supported(const train_config& cfg, const replay* rp_);
unsigned int square_splits(unsigned int Bp, unsigned int H);   // K splits of the dW2 product
hipError_t wide_init_buffers(trainer* t);                       // once, after the workspace is cleared
// bf16 operand copies from padded fp32 parameters (host): of the trained network, or of the target
hipError_t wide_set_weights(trainer* t, const float* padded, bool target);
// Enqueue the step's kernels after the append; `sample` = draw and gather the batch first
// (otherwise X, XT and the per-row fields have been filled by the caller).
hipError_t enqueue_wide_step(trainer* t, hipStream_t st, unsigned int* count, bool sample);
}  // namespace rp
