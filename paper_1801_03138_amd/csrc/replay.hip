// Device-resident FIFO experience replay: storage layout, append, and the
// fused sample + gather + unpack kernels, behind the C entry points replay_*.
//
// Paper: Methods (packed rows of 2D+3 values, add / sample API, FIFO, uniform
// integer sampling with replacement) and Discussion (one state per experience).
#include <mutex>
#include <vector>

#include "common.hpp"
#include "gather_block.hpp"
#include "philox.hpp"
#include "replay_kernels.hpp"

// Scratch of replay_sample_gather_static, the entry point for callers that cannot allocate:
// the slot numbers of one batch without duplicates, between the kernel that draws them and the
// kernel that gathers.  It is part of the library's image, so every GPU the library runs on holds
// its own copy (256 KB) at its own address until the process ends.  In host code the name below
// is only a handle for hipGetSymbolAddress; kernels get the looked-up device address.
constexpr unsigned int kStaticDrawWords = 65536;
static __device__ __align__(256) unsigned int scratch[kStaticDrawWords];

namespace rp {

static thread_local char g_error[512] = "";

char* error_buffer() { return g_error; }

void set_error(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_error, sizeof(g_error), fmt, ap);
    va_end(ap);
}

namespace {

constexpr unsigned int kThreads = kGatherThreads;
constexpr unsigned int kResidentBlocks = 8 * 256;   // blocks of kThreads the chip's 256 compute units hold at once
constexpr unsigned int kMaxPairRowBytes = 32768;  // a gathered PAIR row is staged through LDS

unsigned int elem_bytes_of(unsigned int dtype) { return dtype == RP_F32 ? 4 : dtype == RP_BF16 ? 2 : 1; }

// Stored rows are padded so that 16-byte vector accesses never straddle a row
// and rows of more than 64 bytes start on a 128-byte line.
size_t padded_row(size_t raw) {
    if (raw <= 16) return 16;
    if (raw <= 32) return 32;
    if (raw <= 64) return 64;
    return align_up(raw, 128);
}

struct Layout {
    size_t state_bytes, meta_off, row_bytes;
    size_t off_stage_s, off_stage_s_next, off_stage_a, off_stage_r, off_stage_term;
    size_t off_a, off_r, off_term, off_draw, off_rows, total;
};

bool compute_layout(const replay_config* c, Layout* L) {
    if (!c || c->capacity == 0 || c->capacity >= (1ull << 32) || c->state_dim == 0 ||
        c->state_dim > (1u << 24) || c->state_dtype > RP_U8 || c->layout > RP_CHAIN ||
        c->max_append == 0 || c->max_append > (1u << 24) || c->sampling > RP_DISTINCT ||
        c->reserved != 0)
        return false;
    const size_t eb = elem_bytes_of(c->state_dtype);
    L->state_bytes = (size_t)c->state_dim * eb;
    if (c->layout == RP_PAIR) {
        L->meta_off = align_up(2 * L->state_bytes, 4);
        L->row_bytes = padded_row(L->meta_off + 12);
        if (L->row_bytes > kMaxPairRowBytes) return false;
    } else {
        L->meta_off = 0;
        L->row_bytes = padded_row(L->state_bytes);
    }
    size_t o = 256;  // RingState lives in the first 256 bytes
    auto take = [&](size_t bytes) {
        size_t at = o;
        o = align_up(o + bytes, 256);
        return at;
    };
    const size_t m = c->max_append;
    L->off_stage_s = take(m * L->state_bytes);
    L->off_stage_s_next = take(c->layout == RP_PAIR ? m * L->state_bytes : 0);
    L->off_stage_a = take(m * 4);
    L->off_stage_r = take(m * 4);
    L->off_stage_term = take(m);
    const size_t side = c->layout == RP_CHAIN ? c->capacity : 0;
    L->off_a = take(side * 4);
    L->off_r = take(side * 4);
    L->off_term = take(side);
    // slot numbers of a batch without duplicates, drawn by a kernel of its own ahead of the gather
    // (a batch never holds more members than the replay has experiences)
    L->off_draw = take(c->sampling == RP_DISTINCT ? (size_t)c->capacity * 4 : 0);
    L->off_rows = take((size_t)c->capacity * L->row_bytes);
    L->total = o;
    return true;
}

// PAIR rows, built one 32-bit word per thread.
template <int ELEM>
__global__ __launch_bounds__(kThreads) void append_pair_kernel(AppendArgs p) {
    const RingGeom& g = p.g;
    const unsigned long long n = p.n;
    const unsigned int rows_per_block = p.rows_per_block;
    const unsigned long long head = p.pos.head;
    store_state_after(g, p.pos, n);
    const unsigned int words = g.row_bytes >> 2;
    const unsigned long long row0 = (unsigned long long)blockIdx.x * rows_per_block;
    for (unsigned int e = threadIdx.x; e < rows_per_block * words; e += kThreads) {
        const unsigned int k = e / words, w = e - k * words;
        const unsigned long long row = row0 + k;
        if (row >= n) break;
        unsigned long long slot = head + row;
        if (slot >= g.capacity) slot -= g.capacity;
        const unsigned int val = payload_row_word<ELEM>(g, p.src, row, w);
        reinterpret_cast<unsigned int*>(g.rows + slot * g.row_bytes)[w] = val;
    }
}

// The same for large appends of 2- or 4-byte state elements: a block composes 32 rows in LDS.
// Each source array is read as one contiguous run (consecutive lanes, consecutive elements),
// and the finished rows leave as 16-byte vectors, sixteen lanes per 256-byte row.
template <typename E>
__global__ __launch_bounds__(kThreads) void append_pair_bulk_kernel(AppendArgs p) {
    constexpr unsigned int kRows = 32;
    extern __shared__ uint4 bulk_smem[];
    unsigned char* rows_s = reinterpret_cast<unsigned char*>(bulk_smem);
    const RingGeom& g = p.g;
    const unsigned long long n = p.n, head = p.pos.head;
    store_state_after(g, p.pos, n);
    const unsigned long long row0 = (unsigned long long)blockIdx.x * kRows;
    const unsigned int nrows = (unsigned int)(n - row0 < kRows ? n - row0 : kRows);
    const unsigned int D = g.state_dim, rb = g.row_bytes;
    const E* __restrict__ s = reinterpret_cast<const E*>(p.src.s) + row0 * D;
    const E* __restrict__ sn = reinterpret_cast<const E*>(p.src.s_next) + row0 * D;
    // padding first (bytes between the states and the scalars, and after them)
    for (unsigned int e = threadIdx.x; e < nrows * (rb >> 2); e += kThreads)
        reinterpret_cast<unsigned int*>(rows_s)[e] = 0u;
    __syncthreads();
    for (unsigned int e = threadIdx.x; e < nrows * D; e += kThreads) {
        const unsigned int k = e / D, c = e - k * D;
        E* row = reinterpret_cast<E*>(rows_s + (size_t)k * rb);
        row[c] = s[e];
        row[D + c] = sn[e];
    }
    for (unsigned int k = threadIdx.x; k < nrows; k += kThreads) {
        unsigned int* meta = reinterpret_cast<unsigned int*>(rows_s + (size_t)k * rb + g.meta_off);
        meta[0] = (unsigned int)p.src.a[row0 + k];
        meta[1] = __float_as_uint(p.src.r[row0 + k]);
        meta[2] = p.src.term[row0 + k] ? 1u : 0u;
    }
    __syncthreads();
    const unsigned int V = rb >> 4;
    for (unsigned int e = threadIdx.x; e < nrows * V; e += kThreads) {
        const unsigned int k = e / V, v = e - k * V;
        unsigned long long slot = head + row0 + k;
        if (slot >= g.capacity) slot -= g.capacity;
        reinterpret_cast<u32x4*>(g.rows + slot * rb)[v] =
            reinterpret_cast<const u32x4*>(rows_s + (size_t)k * rb)[v];
    }
}

// CHAIN: one block per experience copies the state into its slot and the three scalars
// into the side arrays.  VEC: state_bytes is a multiple of 16 and the source is 16-byte aligned.
template <bool VEC>
__global__ __launch_bounds__(kThreads) void append_chain_kernel(
    RingGeom g, RingPos pos, unsigned long long n, const unsigned char* __restrict__ s,
    const int* __restrict__ a, const float* __restrict__ r,
    const unsigned char* __restrict__ term) {
    const unsigned long long head = pos.head;
    store_state_after(g, pos, n);
    for (unsigned long long row = blockIdx.x; row < n; row += gridDim.x) {
        unsigned long long slot = head + row;
        if (slot >= g.capacity) slot -= g.capacity;
        unsigned char* dst = g.rows + slot * g.row_bytes;
        const unsigned char* src = s + row * g.state_bytes;
        if (VEC) {
            const unsigned int nv = g.state_bytes >> 4;
            for (unsigned int v = threadIdx.x; v < nv; v += kThreads)
                reinterpret_cast<uint4*>(dst)[v] = reinterpret_cast<const uint4*>(src)[v];
        } else {
            for (unsigned int b = threadIdx.x; b < g.state_bytes; b += kThreads) dst[b] = src[b];
        }
        if (threadIdx.x == 0) {
            g.a[slot] = a[row];
            g.r[slot] = r[row];
            g.term[slot] = term[row] ? 1 : 0;
        }
    }
}

template <int ELEM, int U, int MODE>
__global__ __launch_bounds__(kThreads) void sample_gather_pair_kernel(
    RingGeom g, unsigned long long seed, unsigned long long step_value,
    const unsigned long long* __restrict__ step_ptr, unsigned int size_value, unsigned int batch,
    unsigned int lane_shift, GatherOut out, const unsigned int* __restrict__ drawn) {
    // callers that mirror the ring state pass the size by value: no dependent load up front
    unsigned long long step = 0;
    unsigned int size = 0;
    if (MODE != kDrawGiven) {
        step = step_ptr ? *step_ptr : step_value;
        size = size_value ? size_value : (unsigned int)g.state->size;
    }
    gather_pair_block<ELEM, U, MODE, false>(g, seed, step, size, batch, lane_shift, out,
                                            Payload{nullptr, nullptr, nullptr, nullptr, nullptr}, 0, 0, drawn);
}

// ---------------------------------------------------------------------------------------
// Slot numbers of a batch without duplicates, drawn ahead of the gather into `out` (device
// scratch).  A draw is some sixty dependent Philox blocks, all arithmetic: it wants every lane of
// the chip busy with a draw of its own (G = 0: one draw per lane, 64 per single-wavefront
// workgroup, so that 65,536 draws put one wavefront on each of the chip's 1,024 SIMDs), or, for
// batches too small to fill the chip that way, 2^G lanes per draw that take G rounds at a time
// (distinct_draw_team).  CHAIN rings: the draw counts from the oldest experience and skips the
// newest (it has no successor yet); `out` receives physical slot numbers either way.
// ---------------------------------------------------------------------------------------
template <int G>
__global__ __launch_bounds__(64) void distinct_draw_kernel(
    RingGeom g, unsigned long long seed, unsigned long long step_value,
    const unsigned long long* __restrict__ step_ptr, unsigned int size_value,
    unsigned long long head_value, unsigned int batch, unsigned int* __restrict__ out) {
    __shared__ unsigned int keys[kDistinctTableWords];
    const unsigned int lane = threadIdx.x;
    if (lane < kDistinctTableWords - 64u) keys[64u + lane] = 0u;   // entries no lane computes
    const unsigned long long step = step_ptr ? *step_ptr : step_value;
    const unsigned long long size = size_value ? size_value : g.state->size;
    const unsigned long long head = size_value ? head_value : g.state->head;
    const bool chain = g.layout == RP_CHAIN;
    const unsigned int choices = (unsigned int)(chain ? size - 1 : size);
    const unsigned int rounds = distinct_rounds(choices);
    distinct_round_keys(seed, step, choices, rounds, lane, keys);
    __syncthreads();
    constexpr unsigned int per_block = 64u >> G;
    const unsigned int i = blockIdx.x * per_block + (lane >> G);
    const unsigned int ic = i < batch ? i : batch - 1u;
    unsigned int u;
    if constexpr (G == 0) u = distinct_draw_serial(seed, step, ic, choices, rounds, keys);
    else u = distinct_draw_team<G>(seed, step, ic, choices, rounds, keys, lane);
    if (i < batch && (lane & ((1u << G) - 1u)) == 0) {
        unsigned long long p = u;
        if (chain) {
            unsigned long long oldest = head + g.capacity - size;
            if (oldest >= g.capacity) oldest -= g.capacity;
            p += oldest;
            if (p >= g.capacity) p -= g.capacity;
        }
        out[i] = (unsigned int)p;
    }
}

// The same draw and the gather in one launch (PAIR rings, batches drawn by teams: G > 0): a
// block of four wavefronts draws the 256 >> G slot numbers of its rows into LDS, 2^G lanes per
// draw as above, and gathers those rows, U * (256 >> lane_shift) at a time.  Every lane of the
// block takes part in the draw, and the gather follows without a second launch.  Needs the
// gather's dynamic LDS for one such group of rows.
template <int ELEM, int G, int U>
__global__ __launch_bounds__(kThreads) void sample_gather_pair_distinct_kernel(
    RingGeom g, unsigned long long seed, unsigned long long step_value,
    const unsigned long long* __restrict__ step_ptr, unsigned int size_value, unsigned int batch,
    unsigned int lane_shift, GatherOut out) {
    __shared__ unsigned int keys[kDistinctTableWords];
    __shared__ unsigned int slot_s[kThreads >> G];
    const unsigned int lane = threadIdx.x & 63u;
    const unsigned long long step = step_ptr ? *step_ptr : step_value;
    const unsigned int size = size_value ? size_value : (unsigned int)g.state->size;
    const unsigned int rounds = distinct_rounds(size);
    if (threadIdx.x < 64u) {
        if (lane < kDistinctTableWords - 64u) keys[64u + lane] = 0u;   // entries no lane computes
        distinct_round_keys(seed, step, size, rounds, lane, keys);
    }
    __syncthreads();
    constexpr unsigned int R = kThreads >> G;
    const unsigned int i0 = blockIdx.x * R;
    const unsigned int i = i0 + (threadIdx.x >> G);
    const unsigned int ic = i < batch ? i : batch - 1u;
    unsigned int u;
    if constexpr (G == 0) u = distinct_draw_serial(seed, step, ic, size, rounds, keys);
    else u = distinct_draw_team<G>(seed, step, ic, size, rounds, keys, lane);
    if ((threadIdx.x & ((1u << G) - 1u)) == 0) slot_s[threadIdx.x >> G] = u;
    __syncthreads();
    const unsigned int nrows = min(R, batch - i0);
    const unsigned int group = U * (kThreads >> lane_shift);
    for (unsigned int at = 0; at < nrows; at += group) {
        gather_pair_rows<ELEM, U, kDrawGiven, false>(g, seed, step, size, lane_shift, out,
                                                     Payload{nullptr, nullptr, nullptr, nullptr, nullptr}, 0, 0,
                                                     slot_s, at, i0 + at, min(group, nrows - at));
        __syncthreads();   // (the next group reuses the rows' LDS)
    }
}

// Append, then sample and gather, in one launch (the first kernel of the train steps on MFMA).
template <int ELEM, int MODE>
__global__ __launch_bounds__(kThreads) void append_sample_gather_pair_kernel(AppendGatherArgs p) {
    append_gather_block<ELEM, MODE>(p, blockIdx.x, gridDim.x);
}

// ---------------------------------------------------------------------------------------
// Sample + gather + convert, CHAIN layout (large states).  A block moves one 4 KB piece of
// one state of one sampled experience; s comes from the sampled slot, s' from the slot after
// it.  MODE 0: uint8 -> float with every access coalesced: a wavefront reads 256 contiguous
// bytes as one dword per lane and writes 1 KB as one float4 per lane, four times.
// MODE 1: raw 16-byte copies (float / bf16 states).  MODE 2: element-wise fallback for
// shapes whose rows are not 16-byte multiples.
// ---------------------------------------------------------------------------------------
template <int ELEM, int MODE>
__global__ __launch_bounds__(kThreads) void sample_gather_chain_kernel(
    RingGeom g, unsigned long long seed, unsigned long long step_value,
    const unsigned long long* __restrict__ step_ptr, unsigned int size_value,
    unsigned long long head_value, unsigned int batch, unsigned int chunks,
    void* __restrict__ out_s, void* __restrict__ out_s_next, unsigned int out_ld,
    int* __restrict__ out_a, float* __restrict__ out_r, unsigned char* __restrict__ out_term,
    unsigned int* __restrict__ out_idx, const unsigned int* __restrict__ drawn) {
    const unsigned int chunk = blockIdx.x % chunks;
    const unsigned int t = blockIdx.x / chunks;
    const unsigned int which = t & 1u;
    const unsigned int i = t >> 1;
    if (i >= batch) return;

    unsigned long long p;
    if (drawn) {
        p = drawn[i];   // physical slot numbers, drawn by an earlier kernel
    } else {
        const unsigned long long step = step_ptr ? *step_ptr : step_value;
        const unsigned long long size = size_value ? size_value : g.state->size;
        const unsigned long long head = size_value ? head_value : g.state->head;
        unsigned long long oldest = head + g.capacity - size;
        if (oldest >= g.capacity) oldest -= g.capacity;
        p = oldest + batch_draw(g.sampling, seed, step, i, (unsigned int)(size - 1));
        if (p >= g.capacity) p -= g.capacity;
    }
    unsigned long long q = p;
    if (which) q = (p + 1 == g.capacity) ? 0 : p + 1;

    if (chunk == 0 && which == 0 && threadIdx.x == 0) {
        if (out_idx) out_idx[i] = (unsigned int)p;
        if (out_a) out_a[i] = g.a[p];
        if (out_r) out_r[i] = g.r[p];
        if (out_term) out_term[i] = g.term[p];
    }
    void* out = which ? out_s_next : out_s;
    if (!out) return;
    const unsigned char* src = g.rows + q * g.row_bytes;

    if (MODE == 0) {
        // state_bytes is a multiple of 4 and output rows are 16-byte aligned
        const unsigned int wave = threadIdx.x >> 6, lane = threadIdx.x & 63u;
        const unsigned int base = chunk * 4096u + wave * 1024u + lane * 4u;
        float* dst = static_cast<float*>(out) + (size_t)i * out_ld;
        unsigned int w[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const unsigned int b0 = base + 256u * j;
            w[j] = b0 < g.state_bytes ? *reinterpret_cast<const unsigned int*>(src + b0) : 0u;
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const unsigned int b0 = base + 256u * j;
            if (b0 < g.state_bytes) {
                const float4 f = make_float4(unit_from_u8(w[j] & 0xFFu), unit_from_u8((w[j] >> 8) & 0xFFu),
                                             unit_from_u8((w[j] >> 16) & 0xFFu), unit_from_u8(w[j] >> 24));
                *reinterpret_cast<float4*>(dst + b0) = f;
            }
        }
        return;
    }

    const unsigned int v = chunk * kThreads + threadIdx.x;
    const unsigned int byte0 = v * 16u;
    if (byte0 >= g.state_bytes) return;
    // the slot is padded to a multiple of 16 bytes, so this load stays inside it
    const uint4 val = reinterpret_cast<const uint4*>(src)[v];
    const unsigned int words[4] = {val.x, val.y, val.z, val.w};
    const unsigned int valid_bytes = min(16u, g.state_bytes - byte0);
    constexpr unsigned int EPV = 16 / ELEM;  // elements per 16-byte vector
    const unsigned int e0 = byte0 / ELEM;
    const size_t o = (size_t)i * out_ld + e0;

    if (ELEM == 1) {
        float* dst = static_cast<float*>(out) + o;
#pragma unroll
        for (int j = 0; j < 16; ++j)
            if ((unsigned int)j < valid_bytes)
                dst[j] = unit_from_u8((words[j >> 2] >> (8 * (j & 3))) & 0xFFu);
    } else if (ELEM == 2) {
        unsigned short* dst = static_cast<unsigned short*>(out) + o;
        if (MODE == 1 && valid_bytes == 16) {
            *reinterpret_cast<uint4*>(dst) = val;
        } else {
#pragma unroll
            for (unsigned int j = 0; j < EPV; ++j)
                if (2 * j < valid_bytes)
                    dst[j] = (unsigned short)(words[j >> 1] >> (16 * (j & 1)));
        }
    } else {
        unsigned int* dst = static_cast<unsigned int*>(out) + o;
        if (MODE == 1 && valid_bytes == 16) {
            *reinterpret_cast<uint4*>(dst) = val;
        } else {
#pragma unroll
            for (unsigned int j = 0; j < EPV; ++j)
                if (4 * j < valid_bytes) dst[j] = words[j];
        }
    }
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Device address of `scratch` on GPU `device`, looked up once per GPU with that GPU current.
constexpr int kMaxDevices = 64;
unsigned int* g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mutex;

hipError_t static_scratch_address(int device, unsigned int** out) {
    if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[device]) {
        int current = -1;
        hipError_t e = hipGetDevice(&current);
        if (e != hipSuccess) return e;
        if (current != device) return hipErrorInvalidDevice;   // looked up with its own GPU current only
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        g_scratch_ptr[device] = static_cast<unsigned int*>(p);
    }
    *out = g_scratch_ptr[device];
    return hipSuccess;
}

}  // namespace

AppendArgs make_append_args(const RingGeom& g, const RingPos& pos, unsigned long long n,
                            const Payload& src) {
    AppendArgs a;
    a.g = g;
    a.pos = pos;
    a.n = n;
    a.src = src;
    const unsigned int words = g.row_bytes >> 2;
    a.rows_per_block = kThreads * 4 / words;  // about four words per thread
    if (a.rows_per_block == 0) a.rows_per_block = 1;
    return a;
}

unsigned int append_blocks(const AppendArgs& a) {
    return (unsigned int)((a.n + a.rows_per_block - 1) / a.rows_per_block);
}

// lanes per PAIR row in the gather kernels: enough for one 16-byte piece each, at most the whole block
static unsigned int pair_lane_shift(const RingGeom& g) {
    const unsigned int V = g.row_bytes >> 4;
    unsigned int lane_shift = 0;
    while ((1u << lane_shift) < V && lane_shift < 8) ++lane_shift;
    return lane_shift;
}

AppendGatherArgs make_append_gather_args(const RingGeom& g, const RingPos& pos, unsigned long long n,
                                         const Payload& src, unsigned long long seed,
                                         const unsigned long long* step_ptr, unsigned int batch,
                                         const GatherOut& out) {
    AppendGatherArgs a;
    static_cast<AppendArgs&>(a) = make_append_args(g, pos, n, src);
    a.seed = seed;
    a.step_ptr = step_ptr;
    a.step_value = 0;
    a.batch = batch;
    a.lane_shift = pair_lane_shift(g);
    a.out = out;
    return a;
}

void* append_gather_func(const RingGeom& g) {
    if (g.layout != RP_PAIR || g.elem_bytes == 1) return nullptr;
    const bool distinct = g.sampling == RP_DISTINCT;
    if (g.elem_bytes == 4)
        return distinct ? reinterpret_cast<void*>(append_sample_gather_pair_kernel<4, kDrawDistinct>)
                        : reinterpret_cast<void*>(append_sample_gather_pair_kernel<4, kDrawUniform>);
    return distinct ? reinterpret_cast<void*>(append_sample_gather_pair_kernel<2, kDrawDistinct>)
                    : reinterpret_cast<void*>(append_sample_gather_pair_kernel<2, kDrawUniform>);
}

void append_gather_shape(const AppendGatherArgs& a, unsigned int* blocks, size_t* lds) {
    const unsigned int R = kThreads >> a.lane_shift;   // one row per thread group
    *blocks = (a.batch + R - 1) / R;
    *lds = (a.g.sampling == RP_DISTINCT ? 4 * (size_t)kThreads : 0) + (size_t)R * a.g.row_bytes;
}

void* append_pair_func(const RingGeom& g) {
    if (g.elem_bytes == 4) return reinterpret_cast<void*>(append_pair_kernel<4>);
    if (g.elem_bytes == 2) return reinterpret_cast<void*>(append_pair_kernel<2>);
    return reinterpret_cast<void*>(append_pair_kernel<1>);
}

hipError_t launch_append(const RingGeom& g, const RingPos& pos, unsigned long long n,
                         const void* s, const void* s_next, const int* a, const float* r,
                         const unsigned char* term, hipStream_t stream) {
    if (n == 0) return hipSuccess;
    const unsigned char* sp = static_cast<const unsigned char*>(s);
    const unsigned char* snp = static_cast<const unsigned char*>(s_next);
    if (g.layout == RP_PAIR) {
        AppendArgs args = make_append_args(g, pos, n, Payload{sp, snp, a, r, term});
        if (n >= 1024 && g.elem_bytes >= 2 && g.row_bytes <= 1024) {
            const unsigned int blocks = (unsigned int)((n + 31) / 32);
            const size_t lds = 32 * (size_t)g.row_bytes;
            if (g.elem_bytes == 4)
                hipLaunchKernelGGL(append_pair_bulk_kernel<unsigned int>, dim3(blocks), dim3(kThreads),
                                   lds, stream, args);
            else
                hipLaunchKernelGGL(append_pair_bulk_kernel<unsigned short>, dim3(blocks),
                                   dim3(kThreads), lds, stream, args);
            return hipGetLastError();
        }
        const unsigned int blocks = append_blocks(args);
        void* kargs[] = {&args};
        hipError_t e = hipLaunchKernel(append_pair_func(g), dim3(blocks), dim3(kThreads), kargs, 0,
                                       stream);
        if (e != hipSuccess) return e;
    } else {
        const unsigned int blocks = (unsigned int)(n < 65536 ? n : 65536);
        if ((g.state_bytes & 15u) == 0 && aligned16(s))
            hipLaunchKernelGGL(append_chain_kernel<true>, dim3(blocks), dim3(kThreads), 0, stream,
                               g, pos, n, sp, a, r, term);
        else
            hipLaunchKernelGGL(append_chain_kernel<false>, dim3(blocks), dim3(kThreads), 0, stream,
                               g, pos, n, sp, a, r, term);
    }
    return hipGetLastError();
}

// Lanes per draw of the kernel that draws a batch without duplicates: a whole wavefront per
// draw while that leaves SIMDs idle (1,024 on the chip), sixteen lanes up to four times that, one
// lane beyond (measured cross-over points are of that order; the arithmetic of a draw is the same
// in every shape, only its latency differs).
static int draw_team_log2(unsigned int batch) { return batch <= 1024u ? 6 : batch <= 8192u ? 4 : 0; }

hipError_t launch_distinct_draw(const RingGeom& g, unsigned long long seed, unsigned long long step_value,
                                const unsigned long long* step_ptr, unsigned int batch,
                                unsigned int size_value, unsigned long long head_value,
                                unsigned int* out, hipStream_t stream) {
    const int G = draw_team_log2(batch);
    const unsigned int per_block = 64u >> G;
    const unsigned int blocks = (batch + per_block - 1) / per_block;
#define RP_LAUNCH_DRAW(GG)                                                                        \
    hipLaunchKernelGGL((distinct_draw_kernel<GG>), dim3(blocks), dim3(64), 0, stream, g, seed,   \
                       step_value, step_ptr, size_value, head_value, batch, out)
    if (G == 6) RP_LAUNCH_DRAW(6);
    else if (G == 4) RP_LAUNCH_DRAW(4);
    else RP_LAUNCH_DRAW(0);
#undef RP_LAUNCH_DRAW
    return hipGetLastError();
}

hipError_t launch_sample_gather(const RingGeom& g, unsigned long long seed,
                                unsigned long long step_value,
                                const unsigned long long* step_ptr, unsigned int batch,
                                void* out_s, void* out_s_next, unsigned int out_ld, int* out_a,
                                float* out_r, unsigned char* out_term, unsigned int* out_idx,
                                hipStream_t stream, void* out_s_t, unsigned int out_t_ld,
                                unsigned int size_value, unsigned long long head_value,
                                unsigned int* draw_scratch, unsigned int* launched, bool draw_in_gather) {
    if (launched) *launched = 0;
    if (out_s_t && (g.layout != RP_PAIR || g.elem_bytes == 1)) return hipErrorInvalidValue;
    // A batch without duplicates is drawn by a kernel of its own when the caller has scratch for
    // it, unless the caller allows the draw inside the gather's launch and the batch is one that
    // leaves lanes idle (2^G lanes per draw): beyond that the draws alone keep every SIMD of the
    // chip busy for their whole chain, and a second launch that gathers with eight blocks per
    // compute unit is faster than the same blocks gathering 256 rows each (65,536 rows: 17.5 us
    // against 22.2 us).
    const bool distinct = g.sampling == RP_DISTINCT;
    const bool merged = distinct && draw_in_gather && g.layout == RP_PAIR && draw_team_log2(batch) != 0;
    const unsigned int* drawn = nullptr;
    if (distinct && draw_scratch && !merged) {
        hipError_t e = launch_distinct_draw(g, seed, step_value, step_ptr, batch, size_value, head_value,
                                            draw_scratch, stream);
        if (e != hipSuccess) return e;
        drawn = draw_scratch;
        if (launched) *launched += 1;
    }
    if (merged) {
        // draw and gather in one launch
        const unsigned int lane_shift = pair_lane_shift(g);
        const unsigned int rows_per_pass = kThreads >> lane_shift;
        const int G = draw_team_log2(batch);
        const unsigned int R = kThreads >> G;
        // (a block's 4 or 16 rows are gathered in groups of one row per 2^lane_shift threads)
        const size_t lds = (size_t)rows_per_pass * g.row_bytes;
        const unsigned int blocks = (batch + R - 1) / R;
        const GatherOut out{out_s, out_s_next, out_ld, out_a, out_r, out_term, out_idx, out_s_t, out_t_ld};
#define RP_LAUNCH_DISTINCT(E, GG)                                                                      \
    hipLaunchKernelGGL((sample_gather_pair_distinct_kernel<E, GG, 1>), dim3(blocks), dim3(kThreads),   \
                       lds, stream, g, seed, step_value, step_ptr, size_value, batch, lane_shift, out)
#define RP_LAUNCH_DISTINCT_E(E)                     \
    do {                                            \
        if (G == 6) RP_LAUNCH_DISTINCT(E, 6);       \
        else RP_LAUNCH_DISTINCT(E, 4);              \
    } while (0)
        if (g.elem_bytes == 4) RP_LAUNCH_DISTINCT_E(4);
        else if (g.elem_bytes == 2) RP_LAUNCH_DISTINCT_E(2);
        else RP_LAUNCH_DISTINCT_E(1);
#undef RP_LAUNCH_DISTINCT_E
#undef RP_LAUNCH_DISTINCT
    } else if (g.layout == RP_PAIR) {
        const unsigned int lane_shift = pair_lane_shift(g);
        const unsigned int rows_per_pass = kThreads >> lane_shift;
        // rows per thread: one while all blocks are resident at once (eight per compute unit;
        // measured on 256-byte rows: a second row adds 0.7 us to a block's chain of draw, load
        // and store, which is all a small batch's launch consists of), more for batches that
        // would otherwise come in several waves of blocks (65,536 rows: 8.0 us against 8.5)
        unsigned int U = 1;
        while (U < 4 && (batch + U * rows_per_pass - 1) / (U * rows_per_pass) > kResidentBlocks &&
               (size_t)2 * U * rows_per_pass * g.row_bytes <= 32 * 1024)   // (the rows wait in LDS)
            U *= 2;
        const unsigned int R = U * rows_per_pass;
        const unsigned int blocks = (batch + R - 1) / R;
        const int mode = drawn ? kDrawGiven : distinct ? kDrawDistinct : kDrawUniform;
        const size_t lds = (mode == kDrawDistinct ? 4 * (size_t)U * kThreads : 0) + (size_t)R * g.row_bytes;
        const GatherOut out{out_s, out_s_next, out_ld, out_a, out_r, out_term, out_idx, out_s_t, out_t_ld};
#define RP_LAUNCH_PAIR(E, UU, MM)                                                                  \
    hipLaunchKernelGGL((sample_gather_pair_kernel<E, UU, MM>), dim3(blocks), dim3(kThreads), lds,   \
                       stream, g, seed, step_value, step_ptr, size_value, batch, lane_shift, out, drawn)
#define RP_LAUNCH_PAIR_U(E, UU)                                             \
    do {                                                                   \
        if (mode == kDrawGiven) RP_LAUNCH_PAIR(E, UU, kDrawGiven);         \
        else if (mode == kDrawDistinct) RP_LAUNCH_PAIR(E, UU, kDrawDistinct); \
        else RP_LAUNCH_PAIR(E, UU, kDrawUniform);                          \
    } while (0)
#define RP_LAUNCH_PAIR_E(E)                                                \
    do {                                                                   \
        if (U == 1) RP_LAUNCH_PAIR_U(E, 1);                                \
        else if (U == 2) RP_LAUNCH_PAIR_U(E, 2);                           \
        else RP_LAUNCH_PAIR_U(E, 4);                                       \
    } while (0)
        if (g.elem_bytes == 4)
            RP_LAUNCH_PAIR_E(4);
        else if (g.elem_bytes == 2)
            RP_LAUNCH_PAIR_E(2);
        else
            RP_LAUNCH_PAIR_E(1);
#undef RP_LAUNCH_PAIR_E
#undef RP_LAUNCH_PAIR_U
#undef RP_LAUNCH_PAIR
    } else {
        const unsigned int vectors = (g.state_bytes + 15u) >> 4;
        const unsigned int chunks = (vectors + kThreads - 1) / kThreads;
        const unsigned long long blocks64 = (unsigned long long)batch * 2ull * chunks;
        if (blocks64 > 0x7FFFFFFFull) return hipErrorInvalidValue;
        const unsigned int blocks = (unsigned int)blocks64;
        const unsigned int out_elem = g.elem_bytes == 1 ? 4 : g.elem_bytes;
        const bool vec = ((size_t)out_ld * out_elem) % 16 == 0 && aligned16(out_s) &&
                         aligned16(out_s_next);
#define RP_LAUNCH_CHAIN(E, MODE)                                                                 \
    hipLaunchKernelGGL((sample_gather_chain_kernel<E, MODE>), dim3(blocks), dim3(kThreads), 0,    \
                       stream, g, seed, step_value, step_ptr, size_value, head_value, batch,      \
                       chunks, out_s, out_s_next,                                                 \
                       out_ld, out_a, out_r, out_term, out_idx, drawn)
        if (g.elem_bytes == 4) {
            if (vec) RP_LAUNCH_CHAIN(4, 1); else RP_LAUNCH_CHAIN(4, 2);
        } else if (g.elem_bytes == 2) {
            if (vec) RP_LAUNCH_CHAIN(2, 1); else RP_LAUNCH_CHAIN(2, 2);
        } else {
            if (vec && (g.state_bytes & 3u) == 0) RP_LAUNCH_CHAIN(1, 0); else RP_LAUNCH_CHAIN(1, 2);
        }
#undef RP_LAUNCH_CHAIN
    }
    if (launched) *launched += 1;
    return hipGetLastError();
}

}  // namespace rp

using rp::Layout;

extern "C" {

const char* rp_last_error(void) { return rp::error_buffer(); }
const char* rp_version(void) { return "ingpu_replay 0.1 (gfx950)"; }

size_t replay_storage_bytes(const replay_config* cfg) {
    Layout L;
    return rp::compute_layout(cfg, &L) ? L.total : 0;
}

size_t replay_row_bytes(const replay_config* cfg) {
    Layout L;
    if (!rp::compute_layout(cfg, &L)) return 0;
    return cfg->layout == RP_PAIR ? L.row_bytes : L.row_bytes + 9;
}

rp_status replay_create(const replay_config* cfg, void* dev_storage, size_t bytes,
                        replay_t** out) {
    RP_REQUIRE(cfg && dev_storage && out, "replay_create: null argument");
    Layout L;
    RP_REQUIRE(rp::compute_layout(cfg, &L),
               "replay_create: invalid configuration (capacity 1..2^32-1, state_dim >= 1, "
               "max_append >= 1, PAIR rows at most %u bytes)", rp::kMaxPairRowBytes);
    RP_REQUIRE((reinterpret_cast<uintptr_t>(dev_storage) & 255u) == 0,
               "replay_create: dev_storage must be 256-byte aligned");
    if (bytes < L.total) {
        rp::set_error("replay_create: storage of %zu bytes is smaller than the %zu needed", bytes,
                      L.total);
        return RP_ENOMEM;
    }
    RP_CHECK_HIP(hipMemset(dev_storage, 0, L.total));
    RP_CHECK_HIP(hipDeviceSynchronize());
    int device = -1;
    RP_CHECK_HIP(hipGetDevice(&device));
    {
        // set-up for replay_sample_gather_static: this GPU's address of the static scratch
        unsigned int* unused = nullptr;
        RP_CHECK_HIP(rp::static_scratch_address(device, &unused));
    }
    replay* rp_ = new (std::nothrow) replay();
    if (!rp_) {
        rp::set_error("replay_create: out of host memory");
        return RP_ENOMEM;
    }
    unsigned char* base = static_cast<unsigned char*>(dev_storage);
    rp_->cfg = *cfg;
    rp_->device = device;
    rp_->storage = base;
    rp_->storage_bytes = L.total;
    rp_->stage_s = base + L.off_stage_s;
    rp_->stage_s_next = base + L.off_stage_s_next;
    rp_->stage_a = reinterpret_cast<int*>(base + L.off_stage_a);
    rp_->stage_r = reinterpret_cast<float*>(base + L.off_stage_r);
    rp_->stage_term = base + L.off_stage_term;
    rp_->draw_scratch = cfg->sampling == RP_DISTINCT ? reinterpret_cast<unsigned int*>(base + L.off_draw)
                                                     : nullptr;
    rp::RingGeom& g = rp_->geom;
    g.capacity = cfg->capacity;
    g.state_dim = cfg->state_dim;
    g.elem_bytes = rp::elem_bytes_of(cfg->state_dtype);
    g.state_bytes = (unsigned int)L.state_bytes;
    g.row_bytes = (unsigned int)L.row_bytes;
    g.meta_off = (unsigned int)L.meta_off;
    g.layout = cfg->layout;
    g.dtype = cfg->state_dtype;
    g.sampling = cfg->sampling;
    g.rows = base + L.off_rows;
    g.a = reinterpret_cast<int*>(base + L.off_a);
    g.r = reinterpret_cast<float*>(base + L.off_r);
    g.term = base + L.off_term;
    g.state = reinterpret_cast<rp::RingState*>(base);
    rp_->head = rp_->size = rp_->total = 0;
    // pinned slots for host-sourced appends
    {
        const size_t m = cfg->max_append, sb = L.state_bytes;
        size_t o = 0;
        auto take = [&](size_t nbytes) { size_t at = o; o = rp::align_up(o + nbytes, 16); return at; };
        take(m * sb);
        rp_->pin_off_s_next = take(cfg->layout == RP_PAIR ? m * sb : 0);
        rp_->pin_off_a = take(m * 4);
        rp_->pin_off_r = take(m * 4);
        rp_->pin_off_term = take(m);
        rp_->pin_slot_bytes = rp::align_up(o, 256);
        rp_->pin_host = rp_->pin_dev = nullptr;
        rp_->pin_next = 0;
        for (auto& ev : rp_->pin_event) ev = nullptr;
        for (auto& live : rp_->pin_live) live = false;
        void* hp = nullptr;
        void* dp = nullptr;
        hipError_t e = hipHostMalloc(&hp, rp_->pin_slot_bytes * replay::kHostSlots, hipHostMallocMapped);
        if (e == hipSuccess) {
            rp_->pin_host = static_cast<unsigned char*>(hp);
            e = hipHostGetDevicePointer(&dp, hp, 0);
        }
        for (auto& ev : rp_->pin_event)
            if (e == hipSuccess) e = hipEventCreateWithFlags(&ev, hipEventDisableTiming);
        if (e != hipSuccess) {
            rp::set_error("replay_create: pinned staging slots: %s", hipGetErrorString(e));
            replay_destroy(rp_);
            return RP_EHIP;
        }
        rp_->pin_dev = static_cast<unsigned char*>(dp);
    }
    *out = rp_;
    return RP_OK;
}

rp_status replay_destroy(replay_t* rp_) {
    if (!rp_) return RP_OK;
    for (auto& ev : rp_->pin_event)
        if (ev) (void)hipEventDestroy(ev);
    if (rp_->pin_host) (void)hipHostFree(rp_->pin_host);
    delete rp_;
    return RP_OK;
}

rp_status replay_append(replay_t* rp_, uint64_t n, const void* s, const void* s_next,
                        const int32_t* a, const float* r, const uint8_t* term, int src_is_device,
                        void* hip_stream) {
    RP_REQUIRE(rp_, "replay_append: null handle");
    if (n == 0) return RP_OK;
    RP_REQUIRE(n <= rp_->cfg.capacity, "replay_append: n = %llu exceeds the capacity %llu",
               (unsigned long long)n, (unsigned long long)rp_->cfg.capacity);
    const bool pair = rp_->cfg.layout == RP_PAIR;
    RP_REQUIRE(s && a && r && term && (!pair || s_next), "replay_append: null field array");
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const rp::RingGeom& g = rp_->geom;
    if (src_is_device) {
        RP_CHECK_HIP(rp::launch_append(g, rp::RingPos{rp_->head, rp_->size, rp_->total}, n, s, s_next, a,
                                       r, term, stream));
    } else {
        const size_t sb = g.state_bytes;
        for (uint64_t done = 0; done < n;) {
            const uint64_t m = (n - done < rp_->cfg.max_append) ? n - done : rp_->cfg.max_append;
            // into the next pinned slot; the kernel reads it in place over the host link
            const unsigned int slot = (unsigned int)(rp_->pin_next % replay::kHostSlots);
            if (rp_->pin_live[slot]) RP_CHECK_HIP(hipEventSynchronize(rp_->pin_event[slot]));
            const size_t base = (size_t)slot * rp_->pin_slot_bytes;
            unsigned char* h = rp_->pin_host + base;
            memcpy(h, static_cast<const unsigned char*>(s) + done * sb, m * sb);
            if (pair)
                memcpy(h + rp_->pin_off_s_next, static_cast<const unsigned char*>(s_next) + done * sb, m * sb);
            memcpy(h + rp_->pin_off_a, a + done, m * 4);
            memcpy(h + rp_->pin_off_r, r + done, m * 4);
            memcpy(h + rp_->pin_off_term, term + done, m);
            const unsigned char* d = rp_->pin_dev + base;
            const uint64_t cap = rp_->cfg.capacity;
            const rp::RingPos pos{(rp_->head + done) % cap,
                                  rp_->size + done > cap ? cap : rp_->size + done, rp_->total + done};
            RP_CHECK_HIP(rp::launch_append(g, pos, m, d, d + rp_->pin_off_s_next,
                                           reinterpret_cast<const int*>(d + rp_->pin_off_a),
                                           reinterpret_cast<const float*>(d + rp_->pin_off_r),
                                           d + rp_->pin_off_term, stream));
            RP_CHECK_HIP(hipEventRecord(rp_->pin_event[slot], stream));
            rp_->pin_live[slot] = true;
            rp_->pin_next += 1;
            done += m;
        }
    }
    rp_->total += n;
    rp_->size = rp_->size + n > rp_->cfg.capacity ? rp_->cfg.capacity : rp_->size + n;
    rp_->head = (rp_->head + n) % rp_->cfg.capacity;
    return RP_OK;
}

// replay_sample_gather with the given scratch for the slot numbers of a batch without duplicates
static rp_status sample_gather_with(replay_t* rp_, uint64_t step, uint32_t batch, void* out_s,
                                    void* out_s_next, int32_t* out_a, float* out_r, uint8_t* out_term,
                                    uint32_t* out_idx, void* hip_stream, unsigned int* draw_scratch,
                                    const char* who, bool draw_in_gather = false) {
    RP_REQUIRE(rp_, "%s: null handle", who);
    RP_REQUIRE(batch >= 1 && batch <= (1u << 24), "%s: batch %u not in 1..2^24", who, batch);
    if (rp_->total < rp_->cfg.burn_in) return RP_SKIPPED_BURN_IN;
    // experiences that can be drawn; a batch without duplicates needs at least `batch` of them
    const uint64_t choices = rp_->cfg.layout == RP_CHAIN ? (rp_->size ? rp_->size - 1 : 0) : rp_->size;
    if (choices == 0 || (rp_->cfg.sampling == RP_DISTINCT && choices < batch)) return RP_SKIPPED_BURN_IN;
    RP_CHECK_HIP(rp::launch_sample_gather(rp_->geom, rp_->cfg.seed, step, nullptr, batch, out_s,
                                          out_s_next, rp_->cfg.state_dim, out_a, out_r, out_term,
                                          out_idx, static_cast<hipStream_t>(hip_stream), nullptr, 0,
                                          (unsigned int)rp_->size, rp_->head, draw_scratch, nullptr,
                                          draw_in_gather));
    return RP_OK;
}

rp_status replay_sample_gather(replay_t* rp_, uint64_t step, uint32_t batch, void* out_s,
                               void* out_s_next, int32_t* out_a, float* out_r, uint8_t* out_term,
                               uint32_t* out_idx, void* hip_stream) {
    return sample_gather_with(rp_, step, batch, out_s, out_s_next, out_a, out_r, out_term, out_idx,
                              hip_stream, rp_ ? rp_->draw_scratch : nullptr, "replay_sample_gather", true);
}

rp_status replay_sample_gather_static(replay_t* rp_, uint64_t step, uint32_t batch, void* out_s,
                                      void* out_s_next, int32_t* out_a, float* out_r,
                                      uint8_t* out_term, uint32_t* out_idx, void* hip_stream) {
    RP_REQUIRE(rp_, "replay_sample_gather_static: null handle");
    unsigned int* ptr = nullptr;
    if (rp_->cfg.sampling == RP_DISTINCT) {
        RP_REQUIRE(batch <= kStaticDrawWords,
                   "replay_sample_gather_static: batch %u exceeds the %u slot numbers the static "
                   "scratch holds (use replay_sample_gather)", batch, kStaticDrawWords);
        RP_CHECK_HIP(rp::static_scratch_address(rp_->device, &ptr));
    }
    return sample_gather_with(rp_, step, batch, out_s, out_s_next, out_a, out_r, out_term, out_idx,
                              hip_stream, ptr, "replay_sample_gather_static");
}

rp_status replay_get_state(replay_t* rp_, uint64_t* head, uint64_t* size, uint64_t* total) {
    RP_REQUIRE(rp_, "replay_get_state: null handle");
    rp::RingState st;
    RP_CHECK_HIP(hipDeviceSynchronize());
    RP_CHECK_HIP(hipMemcpy(&st, rp_->geom.state, sizeof(st), hipMemcpyDeviceToHost));
    if (head) *head = st.head;
    if (size) *size = st.size;
    if (total) *total = st.total;
    if (st.head != rp_->head || st.size != rp_->size || st.total != rp_->total) {
        rp::set_error("replay_get_state: device state (%llu,%llu,%llu) != host mirror (%llu,%llu,%llu)",
                      st.head, st.size, st.total, (unsigned long long)rp_->head,
                      (unsigned long long)rp_->size, (unsigned long long)rp_->total);
        return RP_ESTATE;
    }
    return RP_OK;
}

rp_status replay_read_rows(replay_t* rp_, uint64_t first_slot, uint64_t n, void* s, void* s_next,
                           int32_t* a, float* r, uint8_t* term) {
    RP_REQUIRE(rp_, "replay_read_rows: null handle");
    const rp::RingGeom& g = rp_->geom;
    RP_REQUIRE(first_slot < g.capacity && n <= g.capacity, "replay_read_rows: range out of bounds");
    if (n == 0) return RP_OK;
    RP_CHECK_HIP(hipDeviceSynchronize());
    const size_t sb = g.state_bytes, rb = g.row_bytes;
    const uint64_t chunk_rows = 4096;
    std::vector<unsigned char> raw(chunk_rows * rb);
    std::vector<int> ta(chunk_rows);
    std::vector<float> tr(chunk_rows);
    std::vector<unsigned char> tt(chunk_rows);
    for (uint64_t done = 0; done < n;) {
        const uint64_t slot = (first_slot + done) % g.capacity;
        uint64_t m = n - done;
        if (m > chunk_rows) m = chunk_rows;
        if (m > g.capacity - slot) m = g.capacity - slot;  // stop at the wrap point
        RP_CHECK_HIP(hipMemcpy(raw.data(), g.rows + slot * rb, m * rb, hipMemcpyDeviceToHost));
        if (g.layout == RP_CHAIN) {
            RP_CHECK_HIP(hipMemcpy(ta.data(), g.a + slot, m * 4, hipMemcpyDeviceToHost));
            RP_CHECK_HIP(hipMemcpy(tr.data(), g.r + slot, m * 4, hipMemcpyDeviceToHost));
            RP_CHECK_HIP(hipMemcpy(tt.data(), g.term + slot, m, hipMemcpyDeviceToHost));
        }
        for (uint64_t k = 0; k < m; ++k) {
            const unsigned char* row = raw.data() + k * rb;
            if (s) memcpy(static_cast<unsigned char*>(s) + (done + k) * sb, row, sb);
            if (g.layout == RP_PAIR) {
                if (s_next) memcpy(static_cast<unsigned char*>(s_next) + (done + k) * sb, row + sb, sb);
                unsigned int meta[3];
                memcpy(meta, row + g.meta_off, 12);
                if (a) a[done + k] = (int)meta[0];
                if (r) memcpy(&r[done + k], &meta[1], 4);
                if (term) term[done + k] = (uint8_t)meta[2];
            } else {
                if (a) a[done + k] = ta[k];
                if (r) r[done + k] = tr[k];
                if (term) term[done + k] = tt[k];
            }
        }
        done += m;
    }
    return RP_OK;
}

}  // extern "C"
