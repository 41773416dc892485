// Built-in copy engine of the expert cache: pinned host pool -> device slots
// with hipMemcpyAsync on a side stream, one event per slot, and a device
// table of fate_qexpert kept in step with what each slot holds.
//
// Ordering.  Copies alternate between copy_stream and a second stream the
// engine owns (default priority): an expert of a few megabytes does not fill
// the link on its own, two copies in flight hide each other's start-up.
// Before a step the caller hands in the
// event it recorded after the previous layer's FFN; both streams wait for it,
// so a slot released in the previous step is not overwritten while a kernel
// may still read it.  A slot whose last copy was never waited for (an unused
// prefetch) is re-targeted only after a wait for that copy's event on the
// stream of the new copy.  After a step the compute stream waits for the events of
// the slots the current layer uses.  Table entries are written by a one-thread
// kernel on the compute stream (arguments travel by value with the launch).
#include <vector>
#include "common.h"

struct fate_hip_engine {
    int num_layers, E, total_slots;
    fate_slot_layout lay;
    fate_slot_layout lay_low;      // layout of the low-width copies (slot_bytes 0: none)
    char* pool;
    const char* host;
    const char* host_low;
    fate_qexpert* table;
    hipStream_t copy_stream, compute_stream;
    hipStream_t copy2;             // the engine's own second copy stream
    int flip;
    std::vector<hipEvent_t> ev;
    std::vector<uint8_t> ev_live;
    uint64_t bytes;
};

namespace fate {

__global__ void set_entry_kernel(fate_qexpert* dst, fate_qexpert v) {
    if (threadIdx.x == 0 && blockIdx.x == 0) *dst = v;
}

static fate_qexpert entry_for(const fate_hip_engine* g, int slot, const fate_slot_layout& lay) {
    const char* b = g->pool + (size_t)slot * g->lay.slot_bytes;      // slots are spaced by the main layout
    fate_qexpert q;
    q.w1 = b + lay.off_w1; q.w3 = b + lay.off_w3; q.w2 = b + lay.off_w2;
    q.s1 = b + lay.off_s1; q.s3 = b + lay.off_s3; q.s2 = b + lay.off_s2;
    q.bits = lay.bits; q.group = lay.group; q.I = lay.I; q.reserved = 0;
    q.z1 = q.z3 = q.z2 = nullptr; q.reserved2 = 0;      // the pools hold symmetric copies
    return q;
}

}  // namespace fate

using namespace fate;

extern "C" fate_hip_engine* fate_hip_engine_create(int num_layers, int E, int total_slots,
                                                   const fate_slot_layout* layout, void* slot_pool_dev,
                                                   const void* host_pool_pinned, fate_qexpert* table_dev,
                                                   void* copy_stream, void* compute_stream) {
    if (num_layers < 1 || E < 1 || total_slots < 1 || !layout || !slot_pool_dev || !host_pool_pinned ||
        !table_dev || layout->slot_bytes == 0 || (layout->slot_bytes & 15)) {
        set_error("fate_hip_engine_create: bad argument");
        return nullptr;
    }
    const size_t offs[6] = {layout->off_w1, layout->off_w3, layout->off_w2,
                            layout->off_s1, layout->off_s3, layout->off_s2};
    for (size_t o : offs)
        if ((o & 15) || o >= layout->slot_bytes) {
            set_error("fate_hip_engine_create: array offsets must be 16-byte aligned and inside the slot");
            return nullptr;
        }
    fate_hip_engine* g = new fate_hip_engine();
    g->num_layers = num_layers; g->E = E; g->total_slots = total_slots; g->lay = *layout;
    g->pool = static_cast<char*>(slot_pool_dev);
    g->host = static_cast<const char*>(host_pool_pinned);
    g->table = table_dev;
    g->copy_stream = static_cast<hipStream_t>(copy_stream);
    g->compute_stream = static_cast<hipStream_t>(compute_stream);
    g->bytes = 0;
    g->flip = 0;
    g->lay_low = fate_slot_layout{};
    g->host_low = nullptr;
    if (hipStreamCreateWithFlags(&g->copy2, hipStreamNonBlocking) != hipSuccess) {
        delete g;
        set_error("hipStreamCreateWithFlags failed");
        return nullptr;
    }
    g->ev.resize(total_slots);
    g->ev_live.assign(total_slots, 0);
    for (int i = 0; i < total_slots; ++i) {
        if (hipEventCreateWithFlags(&g->ev[i], hipEventDisableTiming) != hipSuccess) {
            for (int j = 0; j < i; ++j) (void)hipEventDestroy(g->ev[j]);
            (void)hipStreamDestroy(g->copy2);
            delete g;
            set_error("hipEventCreateWithFlags failed");
            return nullptr;
        }
    }
    return g;
}

extern "C" void fate_hip_engine_destroy(fate_hip_engine* g) {
    if (!g) return;
    (void)hipStreamSynchronize(g->copy2);
    (void)hipStreamDestroy(g->copy2);
    for (hipEvent_t e : g->ev) (void)hipEventDestroy(e);
    delete g;
}

extern "C" fate_status fate_hip_engine_set_low_pool(fate_hip_engine* g, const fate_slot_layout* layout,
                                                    const void* host_pool_low_pinned) {
    if (!g || !layout || !host_pool_low_pinned || layout->slot_bytes == 0 || (layout->slot_bytes & 15) ||
        layout->slot_bytes > g->lay.slot_bytes || layout->bits == g->lay.bits)
        FATE_FAIL(FATE_EINVAL, "fate_hip_engine_set_low_pool: bad argument");
    const size_t offs[6] = {layout->off_w1, layout->off_w3, layout->off_w2,
                            layout->off_s1, layout->off_s3, layout->off_s2};
    for (size_t o : offs)
        if ((o & 15) || o >= layout->slot_bytes)
            FATE_FAIL(FATE_EINVAL, "array offsets must be 16-byte aligned and inside the slot");
    g->lay_low = *layout;
    g->host_low = static_cast<const char*>(host_pool_low_pinned);
    return FATE_OK;
}

extern "C" int fate_hip_engine_copy(void* engine, int layer, int expert, int slot, int demand, int bits) {
    (void)demand;
    fate_hip_engine* g = static_cast<fate_hip_engine*>(engine);
    if (!g || layer < 0 || layer >= g->num_layers || expert < 0 || expert >= g->E || slot < 0 ||
        slot >= g->total_slots)
        return 1;
    // a width that names the low pool comes from there; every other request is the cache's own copy
    const bool low = g->host_low != nullptr && bits == g->lay_low.bits;
    const fate_slot_layout& lay = low ? g->lay_low : g->lay;
    const char* src = (low ? g->host_low : g->host) + ((size_t)layer * g->E + expert) * lay.slot_bytes;
    const size_t nb = lay.slot_bytes;
    hipStream_t cs = g->flip ? g->copy2 : g->copy_stream;
    g->flip ^= 1;
    // An earlier copy into this slot that nobody waited for (a prefetch that went unused) may
    // still be in flight on the other stream: order this copy after it.
    if (g->ev_live[slot] && hipStreamWaitEvent(cs, g->ev[slot], 0) != hipSuccess) return 5;
    if (hipMemcpyAsync(g->pool + (size_t)slot * g->lay.slot_bytes, src, nb, hipMemcpyHostToDevice, cs) != hipSuccess)
        return 2;
    if (hipEventRecord(g->ev[slot], cs) != hipSuccess) return 3;
    g->ev_live[slot] = 1;
    g->bytes += nb;
    set_entry_kernel<<<1, 64, 0, g->compute_stream>>>(g->table + (size_t)layer * g->E + expert,
                                                     entry_for(g, slot, lay));
    return hipGetLastError() == hipSuccess ? 0 : 4;
}

extern "C" fate_status fate_hip_engine_begin_step(fate_hip_engine* g, void* compute_done_event) {
    if (!g) FATE_FAIL(FATE_EINVAL, "engine is NULL");
    if (compute_done_event) {
        FATE_HIP(hipStreamWaitEvent(g->copy_stream, static_cast<hipEvent_t>(compute_done_event), 0));
        FATE_HIP(hipStreamWaitEvent(g->copy2, static_cast<hipEvent_t>(compute_done_event), 0));
    }
    return FATE_OK;
}

extern "C" fate_status fate_hip_engine_wait_ready(fate_hip_engine* g, const int32_t* slots, int n) {
    if (!g || (n > 0 && !slots)) FATE_FAIL(FATE_EINVAL, "bad argument");
    for (int i = 0; i < n; ++i) {
        const int s = slots[i];
        if (s < 0 || s >= g->total_slots) FATE_FAIL(FATE_EINVAL, "slot %d out of range", s);
        if (g->ev_live[s]) {
            FATE_HIP(hipStreamWaitEvent(g->compute_stream, g->ev[s], 0));
            g->ev_live[s] = 0;
        }
    }
    return FATE_OK;
}

extern "C" fate_status fate_hip_engine_preload(fate_hip_engine* g, int layer, int expert, int slot) {
    if (!g || layer < 0 || layer >= g->num_layers || expert < 0 || expert >= g->E || slot < 0 ||
        slot >= g->total_slots)
        FATE_FAIL(FATE_EINVAL, "bad argument");
    const size_t nb = g->lay.slot_bytes;
    FATE_HIP(hipMemcpy(g->pool + (size_t)slot * nb, g->host + ((size_t)layer * g->E + expert) * nb, nb,
                       hipMemcpyHostToDevice));
    fate_qexpert q = entry_for(g, slot, g->lay);
    FATE_HIP(hipMemcpy(g->table + (size_t)layer * g->E + expert, &q, sizeof(q), hipMemcpyHostToDevice));
    return FATE_OK;
}

extern "C" uint64_t fate_hip_engine_bytes_copied(const fate_hip_engine* g) { return g ? g->bytes : 0; }
