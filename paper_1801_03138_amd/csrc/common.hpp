// Shared host-side plumbing of the library: error reporting and handle layouts.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <cstring>

#include "../../include/ingpu_replay.h"

namespace rp {

// Last failure message of the calling thread.
char* error_buffer();
void set_error(const char* fmt, ...);

#define RP_CHECK_HIP(expr)                                                                  \
    do {                                                                                    \
        hipError_t e_ = (expr);                                                             \
        if (e_ != hipSuccess) {                                                             \
            rp::set_error("%s failed: %s (%s:%d)", #expr, hipGetErrorString(e_), __FILE__,  \
                          __LINE__);                                                        \
            return RP_EHIP;                                                                 \
        }                                                                                   \
    } while (0)

#define RP_REQUIRE(cond, ...)           \
    do {                                \
        if (!(cond)) {                  \
            rp::set_error(__VA_ARGS__); \
            return RP_EINVAL;           \
        }                               \
    } while (0)

#define RP_REQUIRE_STATE(cond, ...)     \
    do {                                \
        if (!(cond)) {                  \
            rp::set_error(__VA_ARGS__); \
            return RP_ESTATE;           \
        }                               \
    } while (0)

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Device-resident replay state.  Kernels read and advance it, so that a
// recorded graph replays correctly; the host keeps a mirror for its decisions.
struct RingState {
    unsigned long long head;   // slot the next experience goes to
    unsigned long long size;   // experiences held
    unsigned long long total;  // experiences ever added
    unsigned int pad_[10];
};
static_assert(sizeof(RingState) == 64, "RingState is one 64-byte line");

// Geometry of the ring in device memory, passed by value to kernels.
struct RingGeom {
    unsigned long long capacity;
    unsigned int state_dim;     // D
    unsigned int elem_bytes;    // 4, 2, 1
    unsigned int state_bytes;   // D * elem_bytes
    unsigned int row_bytes;     // PAIR: padded packed row; CHAIN: padded state slot
    unsigned int meta_off;      // PAIR: byte offset of (action, reward, terminal) in a row
    unsigned int layout;
    unsigned int dtype;
    unsigned int sampling;      // 0: with replacement, 1: without duplicates
    unsigned char* rows;        // PAIR: [capacity][row_bytes]; CHAIN: [capacity][row_bytes] states
    int* a;                     // CHAIN side arrays [capacity]
    float* r;
    unsigned char* term;
    RingState* state;
};

// New experiences handed to a kernel, structure of arrays (device-readable memory).
struct Payload {
    const unsigned char* s;
    const unsigned char* s_next;
    const int* a;
    const float* r;
    const unsigned char* term;
};

// Ring state before an operation, as the host mirrors it: kernels take it by value, so they
// start without a dependent load, and write the state that follows back to device memory.
struct RingPos {
    unsigned long long head, size, total;
};

// Argument block of the PAIR append kernel (one struct, so that a recorded graph node can be
// pointed at another payload by replacing a single kernel argument).
struct AppendArgs {
    RingGeom g;
    unsigned long long n;
    Payload src;
    unsigned int rows_per_block;
    RingPos pos;               // ring state before this append
};

// Where a sample-and-gather launch writes the unpacked batch (see launch_sample_gather).
struct GatherOut {
    void* out_s;
    void* out_s_next;
    unsigned int out_ld;
    int* out_a;
    float* out_r;
    unsigned char* out_term;
    unsigned int* out_idx;
    void* out_s_t;
    unsigned int out_t_ld;
};

// Argument block of the kernel that appends and then samples and gathers in one launch.  It
// starts with the append kernel's block, so one object can feed either kernel.
struct AppendGatherArgs : AppendArgs {
    unsigned long long seed;
    const unsigned long long* step_ptr;   // sampling step (device), or null: step_value then
    unsigned long long step_value;        // (callers that mirror the step pass it by value: no dependent load)
    unsigned int batch, lane_shift;
    GatherOut out;
};

}  // namespace rp

struct replay {
    replay_config cfg;
    int device;                 // the GPU the replay was created on
    rp::RingGeom geom;
    unsigned char* storage;
    size_t storage_bytes;
    // staging area (device) for host-sourced appends, structure of arrays
    unsigned char* stage_s;
    unsigned char* stage_s_next;
    int* stage_a;
    float* stage_r;
    unsigned char* stage_term;
    // scratch for the slot numbers of a batch without duplicates (`capacity` words inside the
    // storage; null for a replay that samples with replacement)
    unsigned int* draw_scratch;
    // host mirror of the ring state
    uint64_t head, size, total;
    // Host-sourced appends: the caller's arrays are copied into one of kHostSlots pinned,
    // device-mapped slots (max_append rows each, structure of arrays) that the append kernel
    // reads in place; an event per slot tells when it may be reused.
    static constexpr unsigned int kHostSlots = 4;
    unsigned char* pin_host;
    unsigned char* pin_dev;
    size_t pin_slot_bytes, pin_off_s_next, pin_off_a, pin_off_r, pin_off_term;
    uint64_t pin_next;
    hipEvent_t pin_event[kHostSlots];
    bool pin_live[kHostSlots];
};
