// Asynchronous weight loading (Section 3.2, "Asynchronous Weight Loading"): host -> device
// copies of the next layer's weight buffer on a copy stream, ordered against the compute
// stream by two events per device slot.  Host code only: no kernel.
// Declarations and the contract of every entry point: include/nimbus_loader.h.
#include <hip/hip_runtime.h>
#include <new>
#include "../../include/nimbus_cop.h"
#include "../../include/nimbus_loader.h"

namespace {

struct Slot {
    hipEvent_t loaded = nullptr;        // recorded on the copy stream after the slot's copy
    hipEvent_t released = nullptr;      // recorded on the compute stream after the last reader
    bool loaded_recorded = false;
    bool released_recorded = false;
};

constexpr int kMaxSlots = 64;

}  // namespace

struct nimbus_loader {
    int slots = 0;
    Slot slot[kMaxSlots];
};

static void destroy_events(nimbus_loader *ld)
{
    for (int i = 0; i < ld->slots; ++i) {
        if (ld->slot[i].loaded) (void)hipEventDestroy(ld->slot[i].loaded);
        if (ld->slot[i].released) (void)hipEventDestroy(ld->slot[i].released);
    }
}

extern "C" {

int nimbus_loader_create(int slots, nimbus_loader **out)
{
    if (!out || slots < 1 || slots > kMaxSlots) return NIMBUS_COP_ERR_INVALID_ARG;
    nimbus_loader *ld = new (std::nothrow) nimbus_loader();
    if (!ld) return NIMBUS_COP_ERR_LAUNCH;
    ld->slots = slots;
    for (int i = 0; i < slots; ++i) {
        // ordering only: no timestamps needed
        if (hipEventCreateWithFlags(&ld->slot[i].loaded, hipEventDisableTiming) != hipSuccess ||
            hipEventCreateWithFlags(&ld->slot[i].released, hipEventDisableTiming) != hipSuccess) {
            destroy_events(ld);
            delete ld;
            (void)hipGetLastError();
            return NIMBUS_COP_ERR_LAUNCH;
        }
    }
    *out = ld;
    return NIMBUS_COP_OK;
}

int nimbus_loader_destroy(nimbus_loader *ld)
{
    if (!ld) return NIMBUS_COP_OK;
    destroy_events(ld);
    delete ld;
    return NIMBUS_COP_OK;
}

int nimbus_loader_load(nimbus_loader *ld, int slot, void *dst_device, const void *src_host,
                       size_t bytes, void *copy_stream)
{
    if (!ld || slot < 0 || slot >= ld->slots || !dst_device || !src_host || bytes == 0)
        return NIMBUS_COP_ERR_INVALID_ARG;
    Slot &s = ld->slot[slot];
    hipStream_t cs = (hipStream_t)copy_stream;
    // the slot's previous contents may still be read by the compute stream
    if (s.released_recorded && hipStreamWaitEvent(cs, s.released, 0) != hipSuccess)
        return NIMBUS_COP_ERR_LAUNCH;
    if (hipMemcpyAsync(dst_device, src_host, bytes, hipMemcpyHostToDevice, cs) != hipSuccess)
        return NIMBUS_COP_ERR_LAUNCH;
    if (hipEventRecord(s.loaded, cs) != hipSuccess) return NIMBUS_COP_ERR_LAUNCH;
    s.loaded_recorded = true;
    return NIMBUS_COP_OK;
}

int nimbus_loader_acquire(nimbus_loader *ld, int slot, void *compute_stream)
{
    if (!ld || slot < 0 || slot >= ld->slots) return NIMBUS_COP_ERR_INVALID_ARG;
    Slot &s = ld->slot[slot];
    if (s.loaded_recorded &&
        hipStreamWaitEvent((hipStream_t)compute_stream, s.loaded, 0) != hipSuccess)
        return NIMBUS_COP_ERR_LAUNCH;
    return NIMBUS_COP_OK;
}

int nimbus_loader_release(nimbus_loader *ld, int slot, void *compute_stream)
{
    if (!ld || slot < 0 || slot >= ld->slots) return NIMBUS_COP_ERR_INVALID_ARG;
    Slot &s = ld->slot[slot];
    if (hipEventRecord(s.released, (hipStream_t)compute_stream) != hipSuccess)
        return NIMBUS_COP_ERR_LAUNCH;
    s.released_recorded = true;
    return NIMBUS_COP_OK;
}

}  // extern "C"
