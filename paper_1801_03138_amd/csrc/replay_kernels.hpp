// Launchers of the replay kernels, shared by the replay entry points and the trainer.
#pragma once

#include "common.hpp"

namespace rp {

// Append n experiences read from device arrays (structure of arrays) to a ring in state
// `pos` (the host mirror's); the kernel also stores the state that follows in device memory.
hipError_t launch_append(const RingGeom& g, const RingPos& pos, unsigned long long n,
                         const void* s, const void* s_next, const int* a, const float* r,
                         const unsigned char* term, hipStream_t stream);

// Pieces of the PAIR append launch, for callers that record it into a graph themselves.
AppendArgs make_append_args(const RingGeom& g, const RingPos& pos, unsigned long long n,
                            const Payload& src);
unsigned int append_blocks(const AppendArgs& a);
void* append_pair_func(const RingGeom& g);   // the __global__ function, as hipLaunchKernel takes it

// Pieces of the launch that appends n experiences and then samples and gathers a batch (PAIR
// rings with 2- or 4-byte elements; the function is null otherwise): argument block, the
// __global__ function, grid size and dynamic LDS bytes.
AppendGatherArgs make_append_gather_args(const RingGeom& g, const RingPos& pos, unsigned long long n,
                                         const Payload& src, unsigned long long seed,
                                         const unsigned long long* step_ptr, unsigned int batch,
                                         const GatherOut& out);
void* append_gather_func(const RingGeom& g);
void append_gather_shape(const AppendGatherArgs& a, unsigned int* blocks, size_t* lds);

// Sample `batch` slots and unpack them.  The sampling step is *step_ptr when
// step_ptr is non-null (device), else step_value.  out_ld is the row pitch of
// out_s / out_s_next in elements (>= D); columns D..out_ld-1 are not written.
// out_s_t (PAIR rings with 2- or 4-byte elements; may be null) receives the old states
// transposed: element (column, i) at out_s_t[column * out_t_ld + i].
// size_value, head_value: the number of experiences held and the write position, when the
// caller mirrors them; size_value = 0 = read both from the device-resident ring state.
// draw_scratch (device, `batch` words; may be null): with it, a batch without duplicates is drawn
// by a kernel of its own into that buffer and the gather reads the slot numbers from there;
// without it the gather kernel draws them itself.  *launched (may be null) receives the number
// of kernels enqueued.
hipError_t launch_sample_gather(const RingGeom& g, unsigned long long seed,
                                unsigned long long step_value,
                                const unsigned long long* step_ptr, unsigned int batch,
                                void* out_s, void* out_s_next, unsigned int out_ld, int* out_a,
                                float* out_r, unsigned char* out_term, unsigned int* out_idx,
                                hipStream_t stream, void* out_s_t = nullptr,
                                unsigned int out_t_ld = 0, unsigned int size_value = 0,
                                unsigned long long head_value = 0, unsigned int* draw_scratch = nullptr,
                                unsigned int* launched = nullptr, bool draw_in_gather = false);

}  // namespace rp
