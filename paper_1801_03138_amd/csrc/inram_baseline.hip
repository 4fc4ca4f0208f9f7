// The comparison system of the paper, re-created: an experience replay kept in host RAM
// (Methods / Results: "in-RAM" replay).  Every train step draws its batch indices on the host,
// gathers the rows into a pinned staging buffer, copies that batch to the GPU and runs the same
// Q-learning step on it (train_step_batch), so the only difference to the device-resident
// replay is where sampling and gathering happen and the per-step host-to-device copy.
// The index stream is the same as the device path's (Philox4x32-10 keyed by seed and step,
// multiply-high map), so both paths train on identical batches.
#include <cstdlib>
#include <new>

#include "common.hpp"

namespace {

// Philox4x32-10 (Salmon et al., SC'11), host version
inline void philox4x32_10_host(uint32_t c[4], uint32_t k0, uint32_t k1) {
    for (int round = 0; round < 10; ++round) {
        const uint64_t p0 = (uint64_t)0xD2511F53u * c[0];
        const uint64_t p1 = (uint64_t)0xCD9E8D57u * c[2];
        const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c[1] ^ k0;
        const uint32_t n1 = (uint32_t)p1;
        const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c[3] ^ k1;
        const uint32_t n3 = (uint32_t)p0;
        c[0] = n0; c[1] = n1; c[2] = n2; c[3] = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
}

constexpr unsigned int kSlots = 16;   // pinned staging batches in flight
constexpr size_t kCopyPiece = 16 * 1024;   // bytes per host-to-device copy call

}  // namespace

struct inram_replay {
    uint64_t capacity, burn_in, seed;
    uint32_t D, batch;
    uint64_t head, size, total, step;
    // ring in ordinary host memory, structure of arrays
    float *s, *s_next, *r;
    int32_t* a;
    uint8_t* term;
    // pinned staging: kSlots batches, each [s | s' | a | r | term] back to back
    unsigned char* pin;
    size_t slot_bytes, off_s_next, off_a, off_r, off_term;
    hipEvent_t copied[kSlots];
    bool live[kSlots];
    uint64_t next_slot;
    unsigned char* dev;   // device buffer of one batch, same layout (caller's memory)
};

extern "C" {

size_t inram_device_bytes(uint32_t state_dim, uint32_t batch) {
    if (state_dim == 0 || batch == 0) return 0;
    size_t o = 0;
    auto take = [&](size_t bytes) { o = rp::align_up(o + bytes, 16); };
    take((size_t)batch * state_dim * 4);
    take((size_t)batch * state_dim * 4);
    take((size_t)batch * 4);
    take((size_t)batch * 4);
    take((size_t)batch);
    return rp::align_up(o, 256);
}

rp_status inram_create(uint64_t capacity, uint32_t state_dim, uint64_t burn_in, uint64_t seed,
                       uint32_t batch, void* dev_batch, size_t bytes, inram_replay_t** out) {
    RP_REQUIRE(out && dev_batch, "inram_create: null argument");
    RP_REQUIRE(capacity >= 1 && capacity < (1ull << 32) && state_dim >= 1 && state_dim <= 4096 &&
                   batch >= 1 && batch <= (1u << 20),
               "inram_create: invalid sizes");
    const size_t need = inram_device_bytes(state_dim, batch);
    if (bytes < need) {
        rp::set_error("inram_create: device buffer of %zu bytes is smaller than the %zu needed", bytes, need);
        return RP_ENOMEM;
    }
    inram_replay* h = new (std::nothrow) inram_replay();
    if (!h) {
        rp::set_error("inram_create: out of host memory");
        return RP_ENOMEM;
    }
    h->capacity = capacity; h->burn_in = burn_in; h->seed = seed; h->D = state_dim; h->batch = batch;
    h->head = h->size = h->total = h->step = 0;
    h->next_slot = 0;
    h->dev = static_cast<unsigned char*>(dev_batch);
    const size_t D = state_dim;
    h->s = static_cast<float*>(malloc(capacity * D * 4));
    h->s_next = static_cast<float*>(malloc(capacity * D * 4));
    h->a = static_cast<int32_t*>(malloc(capacity * 4));
    h->r = static_cast<float*>(malloc(capacity * 4));
    h->term = static_cast<uint8_t*>(malloc(capacity));
    size_t o = 0;
    auto take = [&](size_t nbytes) { size_t at = o; o = rp::align_up(o + nbytes, 16); return at; };
    take((size_t)batch * D * 4);
    h->off_s_next = take((size_t)batch * D * 4);
    h->off_a = take((size_t)batch * 4);
    h->off_r = take((size_t)batch * 4);
    h->off_term = take((size_t)batch);
    h->slot_bytes = rp::align_up(o, 256);
    h->pin = nullptr;
    for (auto& ev : h->copied) ev = nullptr;
    for (auto& l : h->live) l = false;
    void* pin = nullptr;
    hipError_t e = hipHostMalloc(&pin, h->slot_bytes * kSlots, hipHostMallocDefault);
    h->pin = static_cast<unsigned char*>(pin);
    for (auto& ev : h->copied)
        if (e == hipSuccess) e = hipEventCreateWithFlags(&ev, hipEventDisableTiming);
    if (!h->s || !h->s_next || !h->a || !h->r || !h->term || e != hipSuccess) {
        rp::set_error("inram_create: allocation failed (%s)", hipGetErrorString(e));
        inram_destroy(h);
        return e != hipSuccess ? RP_EHIP : RP_ENOMEM;
    }
    *out = h;
    return RP_OK;
}

rp_status inram_destroy(inram_replay_t* h) {
    if (!h) return RP_OK;
    for (auto& ev : h->copied)
        if (ev) (void)hipEventDestroy(ev);
    if (h->pin) (void)hipHostFree(h->pin);
    free(h->s); free(h->s_next); free(h->a); free(h->r); free(h->term);
    delete h;
    return RP_OK;
}

rp_status inram_append(inram_replay_t* h, uint64_t n, const float* s, const float* s_next,
                       const int32_t* a, const float* r, const uint8_t* term) {
    RP_REQUIRE(h, "inram_append: null handle");
    if (n == 0) return RP_OK;
    RP_REQUIRE(n <= h->capacity, "inram_append: n exceeds the capacity");
    RP_REQUIRE(s && s_next && a && r && term, "inram_append: null field array");
    const size_t D = h->D;
    for (uint64_t k = 0; k < n; ++k) {
        const uint64_t slot = (h->head + k) % h->capacity;
        memcpy(h->s + slot * D, s + k * D, D * 4);
        memcpy(h->s_next + slot * D, s_next + k * D, D * 4);
        h->a[slot] = a[k];
        h->r[slot] = r[k];
        h->term[slot] = term[k] ? 1 : 0;
    }
    h->head = (h->head + n) % h->capacity;
    h->size = h->size + n > h->capacity ? h->capacity : h->size + n;
    h->total += n;
    return RP_OK;
}

rp_status inram_train_step(inram_replay_t* h, trainer_t* tr, void* hip_stream) {
    RP_REQUIRE(h && tr, "inram_train_step: null handle");
    if (h->total < h->burn_in || h->size == 0) return RP_SKIPPED_BURN_IN;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const unsigned int slot = (unsigned int)(h->next_slot % kSlots);
    if (h->live[slot]) RP_CHECK_HIP(hipEventSynchronize(h->copied[slot]));
    unsigned char* p = h->pin + (size_t)slot * h->slot_bytes;
    float* ps = reinterpret_cast<float*>(p);
    float* psn = reinterpret_cast<float*>(p + h->off_s_next);
    int32_t* pa = reinterpret_cast<int32_t*>(p + h->off_a);
    float* pr = reinterpret_cast<float*>(p + h->off_r);
    uint8_t* pt = p + h->off_term;
    const size_t D = h->D;
    const uint32_t size = (uint32_t)h->size;
    for (uint32_t i0 = 0; i0 < h->batch; i0 += 4) {
        uint32_t c[4] = {i0 >> 2, 0u, (uint32_t)h->step, (uint32_t)(h->step >> 32)};
        philox4x32_10_host(c, (uint32_t)h->seed, (uint32_t)(h->seed >> 32));
        for (uint32_t j = 0; j < 4 && i0 + j < h->batch; ++j) {
            const uint64_t idx = ((uint64_t)c[j] * size) >> 32;
            const uint32_t i = i0 + j;
            memcpy(ps + i * D, h->s + idx * D, D * 4);
            memcpy(psn + i * D, h->s_next + idx * D, D * 4);
            pa[i] = h->a[idx];
            pr[i] = h->r[idx];
            pt[i] = h->term[idx];
        }
    }
    // The runtime copies up to 16 KB with a kernel on the stream itself (4 us per call); larger
    // transfers take another path that costs 10 us and orders itself against the stream's
    // kernels far more slowly (measured: 65 us per step at batch 128 with one 29 KB copy, 41 us
    // with two copies of half the size; at batch 256, 58 KB, one copy is the faster way, 54 us
    // against 61 us in four).  The comparison system gets the faster way at every size.
    const size_t piece = h->slot_bytes <= 2 * kCopyPiece ? kCopyPiece : h->slot_bytes;
    for (size_t at = 0; at < h->slot_bytes; at += piece) {
        const size_t len = h->slot_bytes - at < piece ? h->slot_bytes - at : piece;
        RP_CHECK_HIP(hipMemcpyAsync(h->dev + at, p + at, len, hipMemcpyHostToDevice, st));
    }
    RP_CHECK_HIP(hipEventRecord(h->copied[slot], st));
    h->live[slot] = true;
    h->next_slot += 1;
    const rp_status s = train_step_batch(tr, h->dev, h->dev + h->off_s_next,
                                         reinterpret_cast<const int32_t*>(h->dev + h->off_a),
                                         reinterpret_cast<const float*>(h->dev + h->off_r),
                                         h->dev + h->off_term, hip_stream);
    if (s < 0) return s;
    h->step += 1;
    return RP_OK;
}

rp_status inram_train_steps(inram_replay_t* h, trainer_t* tr, uint64_t count,
                            uint32_t appends_per_step, const float* s, const float* s_next,
                            const int32_t* a, const float* r, const uint8_t* term, void* hip_stream,
                            uint64_t* executed) {
    RP_REQUIRE(h && tr, "inram_train_steps: null handle");
    uint64_t done = 0;
    const size_t D = h->D;
    for (uint64_t k = 0; k < count; ++k) {
        if (appends_per_step) {
            const uint64_t o = k * appends_per_step;
            const rp_status sa = inram_append(h, appends_per_step, s + o * D, s_next + o * D, a + o,
                                              r + o, term + o);
            if (sa < 0) return sa;
        }
        const rp_status st = inram_train_step(h, tr, hip_stream);
        if (st < 0) {
            if (executed) *executed = done;
            return st;
        }
        done += st == RP_OK;
    }
    if (executed) *executed = done;
    return RP_OK;
}

rp_status inram_get_state(inram_replay_t* h, uint64_t* head, uint64_t* size, uint64_t* total,
                          uint64_t* step) {
    RP_REQUIRE(h, "inram_get_state: null handle");
    if (head) *head = h->head;
    if (size) *size = h->size;
    if (total) *total = h->total;
    if (step) *step = h->step;
    return RP_OK;
}

}  // extern "C"
